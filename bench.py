#!/usr/bin/env python3
"""Benchmark of the PSB layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c1|c3|c4|c4net|c5] [--prob-bits 23|1..7]
                    [--mode product|shared] [--no-cpu-baseline]

A step is one pass of the whole hot path over one batch of synthetic input that is already resident in
HBM: the layer call(s) of the workload through the C-ABI (zero-fill, sampling kernel, fp32 rescale).  The
default workload is benchmark configuration 2 (3x3 conv 64->64 on 1x64x56x56, S=16), the ResNet-shaped layer the
metric is quoted on.  Prints ONE JSON line.

metric  sampled MACs/s: one sampled MAC = one (output element, live tap inside the image, sample)
        shift-add; taps whose activation is 0 are counted (the method as stated samples them), so `value` is
        comparable between implementations whether or not they skip such taps.
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
        instead of 16: 78 units per call.
--mode shared  the shared-filter mode (one sampled filter per pass, the granularity of the paper's simulation;
        reported separately from the headline, which is --mode product).  Its contraction runs on the int8 matrix
        cores: roofline bound "mfma", peak 5.0 POP/s dense int8; achieved = 2 x (output elements) x K x P int8
        operations per launch / kernel time, P = base-256 digit planes of the sampled filter (K = true taps per
        output, padding of the channel count to 32 not counted).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# HBM bytes per launch of the sampling kernel (FETCH_SIZE + WRITE_SIZE of rocprofv3 --pmc, scaled by a 64 MiB copy;
# profiles/k_layer_oc_lane_config2.md).  Measured for the default workload and mapping only.
MEASURED_TRAFFIC_BYTES = {("c2", 0): int((3.9 + 55.4) * (1 << 20))}

# ---- ALU roofline constants (issue rates measured by csrc/valu_rates.hip) ------------------------------
CUS, SIMDS_PER_CU, LANES_PER_SIMD_CLK, CLOCK_HZ = 256, 4, 32, 2.4e9
PEAK_TIOPS = CUS * SIMDS_PER_CU * LANES_PER_SIMD_CLK * CLOCK_HZ / 1e12     # 78.64 T simple int32 lane-ops/s
WIDE = 2                   # units of a half-rate instruction (multiply, three operands, lane-mask producer/consumer)
CALL_UNITS = 15 * WIDE + 31 + 4 * WIDE + 4 * WIDE                          # 77 per generator call (4 samples)
CALL_UNITS_7BIT = 15 * WIDE + 31 + 4 * 4 + 1                               # 78 per generator call (16 samples)
PRODUCT_UNITS = 2 * WIDE                                                   # v_mul_i32_i24 + v_mad_i32_i24
KERNEL_NAMES = {1: "k_layer_pixel_lane", 2: "k_layer_oc_lane", 3: "k_layer_product_list"}
PEAK_INT8_TOPS = 5000.0    # dense int8 MFMA, MI355X


def planes_needed(max_shift, n_samples):
    """Digit planes the library uses for a filter bounded by 2 * n_samples * 2^max_shift (two guard bits)."""
    return min(4, (2 + ((2 * n_samples) << max_shift).bit_length() + 7) // 8)


def shared_ops(L, q):
    """int8 operations (2 per multiply-add) of the shared-filter contraction(s) of one layer call."""
    n, oc = L.x.shape[0], L.w.shape[0]
    oh, ow = L.out_hw
    K = int(np.prod(L.w.shape[1:]))
    max_shift = q.e_top - q.e_min
    if L.budget_to is None:
        return 2.0 * n * oc * oh * ow * K * planes_needed(max_shift, L.S)
    b = np.minimum(L.budget_to, L.s_max)
    levels = sorted(set(np.unique(b).tolist()) | {0})
    ops = 0.0
    for lo, hi in zip(levels[:-1], levels[1:]):
        ops += 2.0 * float((b >= hi).sum()) * oc * K * planes_needed(max_shift, hi - lo)
    return ops


def lane_ops(n_calls, n_products, prob_bits=23):
    """Simple-int32-lane-operation units of n_calls generator calls and n_products products (per lane)."""
    return n_calls * (CALL_UNITS if prob_bits == 23 else CALL_UNITS_7BIT) + n_products * PRODUCT_UNITS


def workload_layers(name):
    from paper_1904_02205_amd import synth
    if name == "c1":
        return [synth.config1()], "config1: linear 512->256, batch 64, uint4 activations, S=8"
    if name == "c2":
        return [synth.config2()], "config2: conv3x3 s1 p1 64->64 on 1x64x56x56 int8 (50% zeros), S=16"
    if name == "c3":
        return [synth.config3()], "config3: progressive conv3x3 128->128 on 8x128x28x28, blob budgets {2..32}"
    if name == "c4":
        return synth.config4_layers(), "config4: 20 convs + FC of a ResNet-18 shape, batch 32, S=8 (layer inputs synthetic)"
    if name == "c4net":
        return None, ("config4 chained: ResNet-18-shaped network end to end, batch 32 at 224x224, S=8, with the glue "
                      "kernels (requantise, residual, pooling) between the layers; synthetic weights and batch norm")
    if name == "c5":
        return synth.config5(), "config5: MobileNet-v2 block at 14x14, batch 64: pruned 1x1 576->160 + depthwise 3x3, S=16"
    raise SystemExit(f"unknown workload {name}")


def count_work(L, packed, torch, device, per_call=4):
    """(sampled MACs, generator calls needed, products needed, sampled MACs with a non-zero activation, dense
    sampled MACs counting padding and dead weights) of one layer call, from the exported weights.

    sampled MACs: sum over outputs of budget x #(live taps inside the image).
    needed: the same restricted to taps whose activation is not 0; calls = ceil(budget/per_call) per such product.
    """
    oc, cin, kh, kw, groups = L.wshape
    cg = cin // groups
    live = ((packed >> 23) & 0xFF) != 0xFF                       # [oc, K]
    live = live.reshape(groups, oc // groups, cg, kh, kw).sum(axis=1).astype(np.float64)   # [g, cg, kh, kw]
    wt = torch.from_numpy(live).to(device)
    x = torch.from_numpy(L.x).to(device)
    ones = torch.ones_like(x, dtype=torch.float64)
    nz = (x != 0).to(torch.float64)
    conv = torch.nn.functional.conv2d
    taps_all = conv(ones, wt, stride=L.stride, padding=L.pad, groups=groups).sum(dim=1)     # [n, oh, ow]
    taps_nz = conv(nz, wt, stride=L.stride, padding=L.pad, groups=groups).sum(dim=1)
    if L.budget_to is not None:
        b = torch.from_numpy(np.minimum(L.budget_to, L.s_max).astype(np.float64)).to(device)
    else:
        b = torch.full_like(taps_all, float(L.S))
    smac = float((taps_all * b).sum().item())
    calls = float((taps_nz * torch.ceil(b / per_call)).sum().item())
    products = float((taps_nz * (b > 0)).sum().item())
    smac_nz = float((taps_nz * b).sum().item())
    dense = float(b.sum().item()) * oc * cg * kh * kw
    return smac, calls, products, smac_nz, dense


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--mapping", type=int, default=0)
    ap.add_argument("--prob-bits", type=int, default=23,
                    help="23 = exact probabilities (the headline metric); 1..7 = discretised, 7-bit uniforms")
    ap.add_argument("--mode", default="product", choices=["product", "shared"],
                    help="product = one random bit per (output, tap, sample), the headline; shared = one sampled "
                         "filter per pass (the paper's simulation granularity)")
    ap.add_argument("--graph", action="store_true",
                    help="c4net only: replay the pass from a captured HIP graph instead of launching it from Python")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-y", action="store_true", help="skip the fp32 rescale output")
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

    layers, desc = workload_layers(args.workload)
    model = None
    if layers is None:
        # the chained network: one pass records every layer's real input, which defines the work that is counted
        from paper_1904_02205_amd import network, resnet_synth, synth
        net = resnet_synth.resnet18(batch=32, hw=224, width=64, classes=1000, device=dev)
        model = network.ResNet18(net, s_max=8, prob_bits=args.prob_bits)
        model.record_inputs = True
        model.forward(S=8, shared=(args.mode == "shared"))
        torch.cuda.synchronize()
        model.record_inputs = False
        layers = []
        for i, sp in enumerate(net.specs):
            x = model.inputs[i].cpu().numpy()
            if x.ndim == 2:
                x = x.reshape(x.shape[0], x.shape[1], 1, 1)
            layers.append(synth.Layer("c4net_" + sp.name, net.weights[i], x, stride=(sp.stride, sp.stride),
                                      pad=(sp.pad, sp.pad), S=8, s_max=8, seed=3, layer_id=i, linear=(sp.name == "fc")))
        model.inputs = {}
    per_call = 4 if args.prob_bits == 23 else 16
    shared = args.mode == "shared"
    calls = []
    kernels = []
    smac = n_calls = n_prod = mfma_ops = smac_nz = smac_dense = 0.0
    for L in layers:
        w = torch.from_numpy(L.w).to(dev)
        q = psb.Weights(w, groups=L.groups, x_absmax=L.x_absmax, s_max=L.s_max, prob_bits=args.prob_bits)
        name = KERNEL_NAMES[psb.query_mapping(q, (L.x.shape[0], L.x.shape[2], L.x.shape[3]) + L.stride + L.pad)]
        if shared:
            name = "k_conv_shared_mfma" if L.groups == 1 and args.mapping != 1 else "k_conv_shared_direct"
            mfma_ops += shared_ops(L, q)
        if name not in kernels:
            kernels.append(name)
        x = torch.from_numpy(L.x).to(dev)
        n, oc = L.x.shape[0], L.w.shape[0]
        oh, ow = L.out_hw
        acc = torch.empty((n, oc, oh, ow), dtype=torch.int32, device=dev)
        y = None if args.no_y else torch.empty((n, oc, oh, ow), dtype=torch.float32, device=dev)
        bt = None if L.budget_to is None else torch.from_numpy(L.budget_to).to(dev)
        packed = q.export()
        if not calls:
            q0_packed = packed
        a, b, c, d, e = count_work(L, packed, torch, dev, per_call)
        smac += a
        n_calls += b
        n_prod += c
        smac_nz += d
        smac_dense += e
        calls.append((L, q, x, acc, y, bt))
    torch.cuda.synchronize()

    graph = None
    if model is not None and args.graph:
        graph, _ = model.capture(S=8, shared=shared)

    def step():
        if graph is not None:
            graph.replay()
            return
        if model is not None:
            model.forward(S=8, shared=shared)
            return
        for L, q, x, acc, y, bt in calls:
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

    if args.copy_calibration:
        src = torch.ones(64 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if graph is not None:
        # launches replayed from a graph run no host code, so the kernels are timed in eager passes beside the
        # timed region (same kernels, same arguments), and the region itself carries no event records
        psb.profile_enable(True)
        psb.profile_read()
        for _ in range(3):
            model.forward(S=8, shared=shared)
        torch.cuda.synchronize()
        kernel_ms, n_launch = psb.profile_read()
        kernel_ms, n_launch = kernel_ms * args.steps / 3, n_launch * args.steps // 3
        psb.profile_enable(False)
    else:
        psb.profile_enable(True)
        psb.profile_read()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    if graph is None:
        kernel_ms, n_launch = psb.profile_read()
        psb.profile_enable(False)

    sec_per_step = (t1 - t0) / args.steps
    value = smac / sec_per_step
    kern_s = kernel_ms * 1e-3 / max(n_launch, 1)                 # average sampling-kernel launch
    launches_per_step = n_launch / args.steps
    ops_per_launch = lane_ops(n_calls, n_prod, args.prob_bits) / launches_per_step
    achieved = ops_per_launch / kern_s / 1e12
    out = {
        "metric": "sampled MACs/sec (int shift-adds/s) on 1 MI355X",
        "value": value, "unit": "sampled MAC/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec_per_step * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": desc, "sampled_macs_per_step": smac,
                   "sampled_macs_with_nonzero_activation_per_step": smac_nz,
                   "sampled_macs_dense_with_padding_per_step": smac_dense,
                   "generator_calls_per_step": n_calls, "samples_per_generator_call": per_call,
                   "prob_bits": args.prob_bits, "mode": args.mode, "hip_graph": bool(args.graph),
                   "kernel_launches_per_step": launches_per_step, "mapping": args.mapping,
                   "rescale_output": not args.no_y,
                   # the network in shared-filter mode runs as one chain: all filters sampled in one launch per pass,
                   # blocked channels-last activations between the convolutions
                   "chained_pass": args.workload == "c4net" and args.mode == "shared"},
        "roofline": {"bound": "alu", "achieved": achieved, "peak": PEAK_TIOPS,
                     "unit": "TIOP/s (simple int32 lane-ops)", "frac": achieved / PEAK_TIOPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, args.mapping))
                     if args.prob_bits == 23 else None,
                     "kernel": "+".join(kernels),
                     "kernel_ms_avg": kern_s * 1e3, "lane_ops_per_launch": ops_per_launch},
    }

    if shared:
        achieved = mfma_ops / launches_per_step / kern_s / 1e12
        out["roofline"] = {"bound": "mfma", "achieved": achieved, "peak": PEAK_INT8_TOPS, "unit": "TOP/s (int8)",
                           "frac": achieved / PEAK_INT8_TOPS, "traffic": None, "kernel": "+".join(kernels),
                           "kernel_ms_avg": kern_s * 1e3, "int8_ops_per_launch": mfma_ops / launches_per_step}

    if not args.no_cpu_baseline:
        from oracle import binding as orc          # the oracle is only timed here, never used for results
        orc.lib()
        L = layers[0]
        qo = orc.QWeights(L.w.reshape(L.w.shape[0], -1), x_absmax=L.x_absmax, s_max=L.s_max,
                          prob_bits=args.prob_bits)
        total = int(np.prod((L.x.shape[0], L.w.shape[0]) + L.out_hw))
        # bounded sample: as many output elements as about 8e9 sampled MACs need, at most all of them
        per_out = smac / sum(np.prod((l.x.shape[0], l.w.shape[0]) + l.out_hw) for l in layers)
        n_pts = int(min(total, max(1000, 8e9 / max(per_out, 1))))
        pts = None if n_pts >= total else np.random.default_rng(0).choice(total, n_pts, replace=False).astype(np.int64)
        c0 = time.perf_counter()
        if shared:
            orc.conv2d_shared(qo, L.wshape, L.x, L.stride, L.pad, S=None if L.budget_to is not None else L.S,
                              s_max=L.s_max, budget_to=L.budget_to, seed=L.seed, layer_id=L.layer_id)
            cpu_smac, pts = smac if len(layers) == 1 else count_work(L, q0_packed, torch, dev, per_call)[0], None
        else:
            _, _, cpu_smac = orc.conv2d(qo, L.wshape, L.x, L.stride, L.pad, S=None if L.budget_to is not None else L.S,
                                        s_max=L.s_max, budget_to=L.budget_to, seed=L.seed, layer_id=L.layer_id,
                                        points=pts)
        c1 = time.perf_counter()
        out["cpu_baseline"] = {"value": cpu_smac / (c1 - c0), "unit": "sampled MAC/s",
                               "cores": orc.num_threads(), "kind": "oracle",
                               "sample": (f"{'all' if pts is None else n_pts} of {total} output elements of "
                                          f"{L.name}, {cpu_smac} sampled MACs, {c1 - c0:.2f} s")}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
