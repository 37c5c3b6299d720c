#!/usr/bin/env python3
"""Benchmark of the PSB layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4|c1|c2|c3|c5|c4net] [--prob-bits 23|1..7] [--per-layer]
                    [--mode product|shared] [--no-per-config] [--no-cpu-baseline]

A step is one pass of the whole hot path over one batch of synthetic input that is already resident in HBM: the
layer call(s) of the workload through the C-ABI (ticket reset / zero-fill, sampling kernel, fp32 rescale).  The
default workload is benchmark configuration 4, the largest one that fits one GPU: the 20 convolutions and the
classifier of a ResNet-18 shape at batch 32, S = 8.  Prints ONE JSON line; with the default workload the line also
carries `per_config`, one record per other configuration (1, 2, 3, 5) measured the same way in the same run.

metric  sampled MACs/s: one sampled MAC = one (output element, live tap inside the image, sample) shift-add; taps
        whose activation is 0 are counted (the method as stated samples them), so `value` is comparable between
        implementations whether or not they skip such taps.
roofline  bound "alu": the sampling kernel is limited by integer VALU issue.  Unit: simple int32 lane-operations
        (a two-operand VALU instruction on vector registers, e.g. v_xor_b32, v_add_u32).  peak = 256 CUs x 4 SIMDs
        x 32 lanes/clock x 2.4 GHz = 78.6 T lane-ops/s (the integer twin of the 157.3 TFLOP/s fp32 vector figure;
        measured: 2.4 cycles per wave64).  Instructions that multiply, take three operands or produce/consume a lane
        mask (v_mad_u64_u32, v_mul_*, v_cmp, v_addc_co) issue at half that rate (measured 4.2-4.5 cycles) and
        count as 2 units.  `achieved` prices only what the method cannot avoid under this keying: per generator
        call (4 samples) 15 wide multiplies, 31 two-input xors (gfx950 has no three-input xor), 4 compares and
        4 carry-adds = 77 units; per product a 24-bit multiply and multiply-add = 4 units; and only for products
        that need sampling (live weight, tap inside the image, activation != 0).  With --prob-bits 1..7 a
        generator call serves 16 samples and its counting is 4 x (or, subtract, and, bit count) + 1 = 17 units
        instead of 16: 78 units per call.  The kernel time is measured live: the library brackets every sampling
        kernel with HIP events on the stream it launches on.
        `traffic`: HBM bytes per launch of the sampling kernel from the rocprofv3 counter summary that is tracked
        under profiles/ for the workload (named in `traffic_source`), null when there is none.
--mode shared  the shared-filter mode (one sampled filter per pass, the granularity of the paper's simulation;
        reported separately from the headline, which is --mode product).  Its contraction runs on the int8 matrix
        cores: roofline bound "mfma", peak 5.0 POP/s dense int8; achieved = 2 x (output elements) x K int8
        operations per launch / kernel time (K = true taps per output): the work of the method.  The kernel
        contracts P base-256 digit planes of the sampled filter; `frac_with_digit_planes` counts P times as much.
"""
import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# rocprofv3 counter summaries with a line "traffic_bytes_per_launch: <int>" (FETCH_SIZE + WRITE_SIZE, scaled by a
# copy of known size), per (workload, mode, prob_bits)
TRAFFIC_PROFILES = {("c4", "product", 23): "profiles/k_layer_oc_lane_config4.md",
                    ("c2", "product", 23): "profiles/k_layer_oc_lane_config2.md",
                    ("c3", "product", 23): "profiles/k_layer_oc_lane_config3.md",
                    ("c5", "product", 23): "profiles/k_layer_product_list_config5.md",
                    ("c4", "shared", 23): "profiles/k_conv_shared_mfma_config4.md",
                    ("c2", "product", 4): "profiles/k_layer_oc_lane_7bit_config2_config4.md#config2",
                    ("c4", "product", 4): "profiles/k_layer_oc_lane_7bit_config2_config4.md#config4"}

# ---- ALU roofline constants (issue rates measured by valu_rates.hip) ------------------------------
CUS, SIMDS_PER_CU, LANES_PER_SIMD_CLK, CLOCK_HZ = 256, 4, 32, 2.4e9
PEAK_TIOPS = CUS * SIMDS_PER_CU * LANES_PER_SIMD_CLK * CLOCK_HZ / 1e12     # 78.64 T simple int32 lane-ops/s
WIDE = 2                   # units of a half-rate instruction (multiply, three operands, lane-mask producer/consumer)
CALL_UNITS = 15 * WIDE + 31 + 4 * WIDE + 4 * WIDE                          # 77 per generator call (4 samples)
CALL_UNITS_7BIT = 15 * WIDE + 31 + 1                                       # 62 per generator call (16 samples) ...
WORD_UNITS_7BIT = 4                                                        # ... + 4 per word of four samples it needs
PRODUCT_UNITS = 2 * WIDE                                                   # v_mul_i32_i24 + v_mad_i32_i24
KERNEL_NAMES = {1: "k_layer_pixel_lane", 2: "k_layer_oc_lane", 3: "k_layer_product_list"}
PEAK_INT8_TOPS = 5000.0    # dense int8 MFMA, MI355X


def planes_needed(max_shift, n_samples):
    """Digit planes the library uses for a filter bounded by 2 * n_samples * 2^max_shift (two guard bits)."""
    return min(4, (2 + ((2 * n_samples) << max_shift).bit_length() + 7) // 8)


def shared_ops(L, q):
    """(int8 operations of the method, the same times the digit planes the kernel contracts) of the shared-filter
    contraction(s) of one layer call; 2 operations per multiply-add."""
    n, oc = L.x.shape[0], L.w.shape[0]
    oh, ow = L.out_hw
    K = int(np.prod(L.w.shape[1:]))
    max_shift = q.e_top - q.e_min
    if L.budget_to is None:
        ops = 2.0 * n * oc * oh * ow * K
        return ops, ops * planes_needed(max_shift, L.S)
    b = np.minimum(L.budget_to, L.s_max)
    levels = sorted(set(np.unique(b).tolist()) | {0})
    ops = planes = 0.0
    for lo, hi in zip(levels[:-1], levels[1:]):
        seg = 2.0 * float((b >= hi).sum()) * oc * K
        ops += seg
        planes += seg * planes_needed(max_shift, hi - lo)
    return ops, planes


def lane_ops(n_calls, n_products, prob_bits=23, n_words=None):
    """Simple-int32-lane-operation units of n_calls generator calls and n_products products (per lane).
    n_words (7-bit uniforms): the words of four samples those calls have to compare (a budget of 8 needs two of a
    call's four); None = four per call."""
    if prob_bits >= 8:
        return n_calls * CALL_UNITS + n_products * PRODUCT_UNITS
    if n_words is None:
        n_words = 4 * n_calls
    return n_calls * CALL_UNITS_7BIT + n_words * WORD_UNITS_7BIT + n_products * PRODUCT_UNITS


WORKLOADS = {
    "c1": "config1: linear 512->256, batch 64, uint4 activations, S=8",
    "c2": "config2: conv3x3 s1 p1 64->64 on 1x64x56x56 int8 (50% zeros), S=16",
    "c3": "config3: progressive conv3x3 128->128 on 8x128x28x28, blob budgets {2..32}",
    "c4": "config4: 20 convs + FC of a ResNet-18 shape, batch 32, S=8 (layer inputs synthetic)",
    "c4net": ("config4 chained: ResNet-18-shaped network end to end, batch 32 at 224x224, S=8, with the glue "
              "kernels (requantise, residual, pooling) between the layers; synthetic weights and batch norm"),
    "c5": "config5: MobileNet-v2 block at 14x14, batch 64: pruned 1x1 576->160 + depthwise 3x3, S=16",
}


def workload_layers(name):
    from paper_1904_02205_amd import synth
    if name not in WORKLOADS:
        raise SystemExit(f"unknown workload {name}")
    layers = {"c1": lambda: [synth.config1()], "c2": lambda: [synth.config2()], "c3": lambda: [synth.config3()],
              "c4": synth.config4_layers, "c5": synth.config5, "c4net": lambda: None}[name]()
    return layers, WORKLOADS[name]


def count_work(L, packed, per_call=4):
    """(sampled MACs, generator calls needed, products needed, sampled MACs with a non-zero activation, dense
    sampled MACs counting padding and dead weights, words of four samples needed) of one layer call, from the
    exported weights.  Host arithmetic.

    sampled MACs: sum over outputs of budget x #(live taps inside the image).
    needed: the same restricted to taps whose activation is not 0; calls = ceil(budget/per_call) per such product.
    """
    oc, cin, kh, kw, groups = L.wshape
    cg = cin // groups
    live = ((packed >> 23) & 0xFF) != 0xFF                                        # [oc, K]
    live = live.reshape(groups, oc // groups, cg, kh, kw).sum(axis=1)             # [g, cg, kh, kw]: channels per tap
    live = live.reshape(cin, kh, kw).astype(np.float32)                           # per input channel
    n, _, h, w = L.x.shape
    oh, ow = L.out_hw
    (sh, sw), (ph, pw) = L.stride, L.pad
    nz = np.zeros((n, cin, h + 2 * ph, w + 2 * pw), dtype=np.float32)
    nz[:, :, ph:ph + h, pw:pw + w] = L.x != 0
    taps_nz = np.zeros((n, oh, ow), dtype=np.float32)         # integers below 2^24: exact in binary32
    taps_all = np.zeros((oh, ow), dtype=np.float64)
    oy, ox = np.arange(oh) * sh - ph, np.arange(ow) * sw - pw
    for a in range(kh):
        row_ok = ((oy + a >= 0) & (oy + a < h)).astype(np.float64)
        for b in range(kw):
            col_ok = ((ox + b >= 0) & (ox + b < w)).astype(np.float64)
            taps_all += float(live[:, a, b].sum()) * np.outer(row_ok, col_ok)
            view = nz[:, :, a:a + sh * (oh - 1) + 1:sh, b:b + sw * (ow - 1) + 1:sw]
            taps_nz += np.einsum("nchw,c->nhw", view, live[:, a, b], optimize=True)
    assert float(live.sum()) < 2 ** 24                        # the largest possible count of one pixel
    taps_nz = taps_nz.astype(np.float64)
    if L.budget_to is not None:
        b = np.minimum(L.budget_to, L.s_max).astype(np.float64)
    else:
        b = np.full((n, oh, ow), float(L.S))
    smac = float((taps_all[None] * b).sum())
    calls = float((taps_nz * np.ceil(b / per_call)).sum())
    products = float((taps_nz * (b > 0)).sum())
    smac_nz = float((taps_nz * b).sum())
    dense = float(b.sum()) * oc * cg * kh * kw
    words = float((taps_nz * np.ceil(b / 4)).sum())
    return smac, calls, products, smac_nz, dense, words


def traffic_of(workload, mode, prob_bits):
    """(bytes per launch, file) from the tracked counter summary of this workload, or (None, None)."""
    rel = TRAFFIC_PROFILES.get((workload, mode, prob_bits))
    if rel is None:
        return None, None
    rel, _, part = rel.partition("#")        # a summary of several workloads has one line per workload
    if not os.path.exists(os.path.join(ROOT, rel)):
        return None, None
    key = "traffic_bytes_per_launch" + ("_" + part if part else "")
    m = re.search(key + r":\s*([0-9][0-9,_]*)", open(os.path.join(ROOT, rel)).read())
    return (int(m.group(1).replace(",", "").replace("_", "")), rel) if m else (None, None)


class Prepared:
    pass


def prepare(workload, args, torch, psb, dev):
    """Tensors in HBM, handles, and the work counts of one workload."""
    P = Prepared()
    P.workload, P.prob_bits, P.mode, P.mapping = workload, args.prob_bits, args.mode, args.mapping
    layers, P.desc = workload_layers(workload)
    P.model = None
    shared = args.mode == "shared"
    if layers is None:
        # the chained network: one pass records every layer's real input, which defines the work that is counted
        from paper_1904_02205_amd import network, resnet_synth, synth
        net = resnet_synth.resnet18(batch=32, hw=224, width=64, classes=1000, device=dev)
        P.model = network.ResNet18(net, s_max=8, prob_bits=args.prob_bits)
        P.model.record_inputs = True
        P.model.forward(S=8, shared=shared)
        torch.cuda.synchronize()
        P.model.record_inputs = False
        layers = []
        for i, sp in enumerate(net.specs):
            x = P.model.inputs[i].cpu().numpy()
            if x.ndim == 2:
                x = x.reshape(x.shape[0], x.shape[1], 1, 1)
            layers.append(synth.Layer("c4net_" + sp.name, net.weights[i], x, stride=(sp.stride, sp.stride),
                                      pad=(sp.pad, sp.pad), S=8, s_max=8, seed=3, layer_id=i, linear=(sp.name == "fc")))
        P.model.inputs = {}
    P.layers = layers
    P.per_call = 4 if args.prob_bits >= 8 else 16
    P.calls, P.kernels, P.layer_smac, P.layer_work = [], [], [], []
    P.smac = P.n_calls = P.n_prod = P.n_words = P.mfma_ops = P.mfma_plane_ops = P.smac_nz = P.smac_dense = 0.0
    for L in layers:
        w = torch.from_numpy(L.w).to(dev)
        q = psb.Weights(w, groups=L.groups, x_absmax=L.x_absmax, s_max=L.s_max, prob_bits=args.prob_bits)
        name = KERNEL_NAMES[psb.query_mapping(q, (L.x.shape[0], L.x.shape[2], L.x.shape[3]) + L.stride + L.pad)]
        if shared:
            # matrix-core contraction: 3 x 3 / stride 1 / padding 1 layers normally run in k_conv3x3_window (both operands
            # from LDS), the others in k_conv_shared_mfma; the library's timer covers whichever it launched
            window = L.w.shape[2:] == (3, 3) and L.stride == (1, 1) and L.pad == (1, 1)
            name = ("k_conv3x3_window" if window else "k_conv_shared_mfma") if L.groups == 1 and args.mapping != 1 \
                else "k_conv_shared_direct"
            a, b = shared_ops(L, q)
            P.mfma_ops += a
            P.mfma_plane_ops += b
        if name not in P.kernels:
            P.kernels.append(name)
        x = torch.from_numpy(L.x).to(dev)
        n, oc = L.x.shape[0], L.w.shape[0]
        oh, ow = L.out_hw
        acc = torch.empty((n, oc, oh, ow), dtype=torch.int32, device=dev)
        y = None if args.no_y else torch.empty((n, oc, oh, ow), dtype=torch.float32, device=dev)
        bt = None if L.budget_to is None else torch.from_numpy(L.budget_to).to(dev)
        a, b, c, d, e, f = count_work(L, q.export(), P.per_call)
        P.n_words += f
        P.smac += a
        P.n_calls += b
        P.n_prod += c
        P.smac_nz += d
        P.smac_dense += e
        P.layer_smac.append(a)
        P.layer_work.append((b, c, f))
        P.calls.append((L, q, x, acc, y, bt))
    torch.cuda.synchronize()
    P.graph = None
    if P.model is not None and args.graph:
        P.graph, _ = P.model.capture(S=8, shared=shared)
    return P


def measure(P, steps, warmup, torch, psb):
    """Time `steps` steps after `warmup` untimed ones; the sampling kernels are timed by the library's HIP events."""
    shared = P.mode == "shared"

    def step():
        if P.graph is not None:
            P.graph.replay()
            return
        if P.model is not None:
            P.model.forward(S=8, shared=shared)
            return
        for L, q, x, acc, y, bt in P.calls:
            if bt is not None:
                psb.conv2d_progressive(q, x, bt, None, stride=L.stride, pad=L.pad, seed=L.seed, layer_id=L.layer_id,
                                       acc=acc, y=y, shared=shared)
            elif L.linear:
                psb.linear(q, x.reshape(x.shape[0], -1), L.S, seed=L.seed, layer_id=L.layer_id,
                           acc=acc.reshape(acc.shape[0], -1), y=None if y is None else y.reshape(y.shape[0], -1),
                           shared=shared)
            else:
                psb.conv2d(q, x, L.S, stride=L.stride, pad=L.pad, seed=L.seed, layer_id=L.layer_id, acc=acc, y=y,
                           shared=shared)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    if P.graph is not None:
        # launches replayed from a graph run no host code, so the kernels are timed in eager passes beside the
        # timed region (same kernels, same arguments), and the region itself carries no event records
        psb.profile_enable(True)
        psb.profile_read()
        for _ in range(3):
            P.model.forward(S=8, shared=shared)
        torch.cuda.synchronize()
        kernel_ms, n_launch = psb.profile_read()
        kernel_ms, n_launch = kernel_ms * steps / 3, n_launch * steps // 3
        psb.profile_enable(False)
    else:
        psb.profile_enable(True)
        psb.profile_read()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    if P.graph is None:
        kernel_ms, n_launch = psb.profile_read()
        psb.profile_enable(False)

    sec_per_step = (t1 - t0) / steps
    kern_s = kernel_ms * 1e-3 / max(n_launch, 1)                 # average sampling-kernel launch
    launches_per_step = n_launch / steps
    traffic, traffic_source = traffic_of(P.workload, P.mode, P.prob_bits)
    if P.mapping != 0:
        traffic, traffic_source = None, None
    if shared:
        achieved = P.mfma_ops / launches_per_step / kern_s / 1e12
        with_planes = P.mfma_plane_ops / launches_per_step / kern_s / 1e12
        roofline = {"bound": "mfma", "achieved": achieved, "peak": PEAK_INT8_TOPS, "unit": "TOP/s (int8)",
                    "frac": achieved / PEAK_INT8_TOPS, "traffic": traffic, "traffic_source": traffic_source,
                    "kernel": "+".join(P.kernels), "kernel_ms_avg": kern_s * 1e3,
                    "int8_ops_per_launch": P.mfma_ops / launches_per_step,
                    "frac_with_digit_planes": with_planes / PEAK_INT8_TOPS}
    else:
        ops_per_launch = lane_ops(P.n_calls, P.n_prod, P.prob_bits, P.n_words) / launches_per_step
        achieved = ops_per_launch / kern_s / 1e12
        roofline = {"bound": "alu", "achieved": achieved, "peak": PEAK_TIOPS,
                    "unit": "TIOP/s (simple int32 lane-ops)", "frac": achieved / PEAK_TIOPS,
                    "traffic": traffic, "traffic_source": traffic_source, "kernel": "+".join(P.kernels),
                    "kernel_ms_avg": kern_s * 1e3, "lane_ops_per_launch": ops_per_launch}
    return {"ms_per_step": sec_per_step * 1e3, "value": P.smac / sec_per_step,
            "launches_per_step": launches_per_step, "roofline": roofline}


def per_layer(P, torch, psb, reps=5):
    """Per-product mode: every layer of the workload on its own - sampling-kernel time (the library's HIP events),
    its share of the ALU roofline and the time a SIMD spends per wave-level generator call."""
    rows = []
    for (L, q, x, acc, y, bt), smac, (calls, prods, words) in zip(P.calls, P.layer_smac, P.layer_work):
        def call():
            if bt is not None:
                psb.conv2d_progressive(q, x, bt, None, stride=L.stride, pad=L.pad, seed=L.seed, layer_id=L.layer_id,
                                       acc=acc, y=y)
            elif L.linear:
                psb.linear(q, x.reshape(x.shape[0], -1), L.S, seed=L.seed, layer_id=L.layer_id,
                           acc=acc.reshape(acc.shape[0], -1), y=None if y is None else y.reshape(y.shape[0], -1))
            else:
                psb.conv2d(q, x, L.S, stride=L.stride, pad=L.pad, seed=L.seed, layer_id=L.layer_id, acc=acc, y=y)
        call()
        torch.cuda.synchronize()
        psb.profile_enable(True)
        psb.profile_read()
        for _ in range(reps):
            call()
        torch.cuda.synchronize()
        ms, n = psb.profile_read()
        psb.profile_enable(False)
        kern_s = ms / max(n, 1) * 1e-3
        rows.append({"layer": L.name, "x": list(L.x.shape), "w": list(L.w.shape), "S": L.S,
                     "kernel_ms": kern_s * 1e3, "sampled_macs_per_s": smac / kern_s,
                     "frac": lane_ops(calls, prods, P.prob_bits, words) / kern_s / 1e12 / PEAK_TIOPS,
                     "ns_per_wave_call_per_simd": kern_s * 1e9 / (calls / 64 / (CUS * SIMDS_PER_CU))})
    return rows


def cpu_baseline(P, budget_smac=1.2e10):
    """The oracle, as it stands, on a bounded sample of the workload: for every layer of it as many randomly chosen
    output elements as an equal share of `budget_smac` sampled MACs needs (all of them if that is fewer)."""
    from oracle import binding as orc          # the oracle is only timed here, never used for results
    orc.lib()
    shared = P.mode == "shared"
    rng = np.random.default_rng(0)
    jobs, n_total, n_used = [], 0, 0
    for L, share in zip(P.layers, P.layer_smac):
        total = int(np.prod((L.x.shape[0], L.w.shape[0]) + L.out_hw))
        per_out = share / total
        n_pts = int(min(total, max(64, budget_smac / len(P.layers) / max(per_out, 1.0))))
        pts = None if n_pts >= total else np.sort(rng.choice(total, n_pts, replace=False)).astype(np.int64)
        qo = orc.QWeights(L.w.reshape(L.w.shape[0], -1), x_absmax=L.x_absmax, s_max=L.s_max, prob_bits=P.prob_bits)
        jobs.append((L, qo, pts))
        n_total += total
        n_used += n_pts
    done = 0.0
    c0 = time.perf_counter()
    for L, qo, pts in jobs:
        kw = dict(S=None if L.budget_to is not None else L.S, s_max=L.s_max, budget_to=L.budget_to, seed=L.seed,
                  layer_id=L.layer_id, points=pts)
        if shared:
            orc.conv2d_shared(qo, L.wshape, L.x, L.stride, L.pad, **kw)
        else:
            _, _, smac = orc.conv2d(qo, L.wshape, L.x, L.stride, L.pad, **kw)
            done += smac
    c1 = time.perf_counter()
    if shared:      # the shared-filter oracle does not count: the same share of the workload's sampled MACs
        done = sum(share * (1.0 if pts is None else pts.size / np.prod((L.x.shape[0], L.w.shape[0]) + L.out_hw))
                   for (L, _, pts), share in zip(jobs, P.layer_smac))
    return {"value": done / (c1 - c0), "unit": "sampled MAC/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": (f"{n_used} of {n_total} output elements, drawn at random from every one of the "
                       f"{len(jobs)} layer(s) of the workload: {done:.4g} sampled MACs in {c1 - c0:.2f} s")}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c4")
    ap.add_argument("--mapping", type=int, default=0)
    ap.add_argument("--prob-bits", type=int, default=23,
                    help="23 = exact probabilities (the headline metric); 8..22 = discretised, 32-bit uniforms; 1..7 = discretised, "
                         "7-bit uniforms")
    ap.add_argument("--mode", default="product", choices=["product", "shared"],
                    help="product = one random bit per (output, tap, sample), the headline; shared = one sampled "
                         "filter per pass (the paper's simulation granularity)")
    ap.add_argument("--graph", action="store_true",
                    help="c4net only: replay the pass from a captured HIP graph instead of launching it from Python")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true",
                    help="default workload only: skip the records of configurations 1, 2, 3 and 5")
    ap.add_argument("--no-y", action="store_true", help="skip the fp32 rescale output")
    ap.add_argument("--per-layer", action="store_true",
                    help="per-product mode, configurations 1-5: add a record of every layer of the workload on its own")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 64 MiB device-to-device copy (reference dispatch for FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every box has one); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    from paper_1904_02205_amd import psb
    psb.lib()
    psb.set_mapping(args.mapping)
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if args.copy_calibration:
        src = torch.ones(64 << 20, dtype=torch.int8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    P = prepare(args.workload, args, torch, psb, dev)
    m = measure(P, args.steps, args.warmup, torch, psb)
    out = {
        "metric": "sampled MACs/sec (int shift-adds/s) on 1 MI355X",
        "value": m["value"], "unit": "sampled MAC/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": m["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": P.desc, "sampled_macs_per_step": P.smac,
                   "sampled_macs_with_nonzero_activation_per_step": P.smac_nz,
                   "sampled_macs_dense_with_padding_per_step": P.smac_dense,
                   "generator_calls_per_step": P.n_calls, "samples_per_generator_call": P.per_call,
                   "prob_bits": args.prob_bits, "mode": args.mode, "hip_graph": bool(args.graph),
                   "kernel_launches_per_step": m["launches_per_step"], "mapping": args.mapping,
                   "rescale_output": not args.no_y,
                   # the network in shared-filter mode runs as one chain: all filters sampled in one launch per pass,
                   # blocked channels-last activations between the convolutions
                   "chained_pass": args.workload == "c4net" and args.mode == "shared"},
        "roofline": m["roofline"],
    }
    if args.per_layer and args.mode == "product" and P.model is None:
        out["per_layer"] = per_layer(P, torch, psb)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(P)
    if args.workload == "c4" and not args.no_per_config:
        del P
        torch.cuda.empty_cache()
        out["per_config"] = []
        for name in ("c1", "c2", "c3", "c5"):
            Pc = prepare(name, args, torch, psb, dev)
            mc = measure(Pc, args.steps, args.warmup, torch, psb)
            r = mc["roofline"]
            out["per_config"].append({"workload": Pc.desc, "ms_per_step": mc["ms_per_step"], "value": mc["value"],
                                      "kernel": r["kernel"], "kernel_ms_avg": r["kernel_ms_avg"],
                                      "launches_per_step": mc["launches_per_step"], "achieved": r["achieved"],
                                      "frac": r["frac"], "traffic": r["traffic"], "traffic_source": r["traffic_source"],
                                      "sampled_macs_per_step": Pc.smac})
            del Pc
    print(json.dumps(out))


if __name__ == "__main__":
    main()
