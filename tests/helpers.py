"""Run one synthetic layer through the CPU oracle / through the HIP library (tests only)."""
import numpy as np


def oracle_quantize(orc, L, exp_bits=0, prob_bits=23):
    w = L.w.reshape(L.w.shape[0], -1)
    return orc.QWeights(w, exp_bits=exp_bits, x_absmax=L.x_absmax, s_max=L.s_max, prob_bits=prob_bits)


def oracle_layer(orc, L, q=None, budget_to=None, budget_from=None, acc_in=None, points=None, S=None, shared=False):
    """acc (int32 [n, oc, oh, ow] or [len(points)]), overflow count, sampled MACs (None in shared-filter mode)."""
    if q is None:
        q = oracle_quantize(orc, L)
    if budget_to is None:
        budget_to = L.budget_to
    S = (L.S if S is None else S) if budget_to is None else None
    if shared:
        acc, over = orc.conv2d_shared(q, L.wshape, L.x, L.stride, L.pad, S=S, s_max=L.s_max, budget_to=budget_to,
                                      budget_from=budget_from, seed=L.seed, layer_id=L.layer_id, acc_in=acc_in,
                                      points=points)
        return acc, over, None
    return orc.conv2d(q, L.wshape, L.x, L.stride, L.pad, S=S, s_max=L.s_max, budget_to=budget_to,
                      budget_from=budget_from, seed=L.seed, layer_id=L.layer_id, points=points, acc_in=acc_in)


def gpu_quantize(psb, L, exp_bits=0, prob_bits=23, device="cuda"):
    import torch
    w = torch.from_numpy(L.w).to(device)
    return psb.Weights(w, groups=L.groups, exp_bits=exp_bits, x_absmax=L.x_absmax, s_max=L.s_max,
                       prob_bits=prob_bits)


def gpu_layer(psb, L, q=None, budget_to=None, budget_from=None, acc_in=None, S=None, want_y=False, mult=None,
              bias=None, device="cuda", shared=False):
    """Returns acc (numpy int32) and y (numpy float32 or None), through the C-ABI entry point the layer names."""
    import torch
    if q is None:
        q = gpu_quantize(psb, L, device=device)
    x = torch.from_numpy(L.x).to(device)
    if budget_to is None:
        budget_to = L.budget_to
    oc = L.w.shape[0]
    oh, ow = L.out_hw
    n = L.x.shape[0]
    acc = None
    if acc_in is not None:
        acc = torch.from_numpy(np.ascontiguousarray(acc_in)).to(device)
    y = torch.empty((n, oc, oh, ow), dtype=torch.float32, device=device) if want_y else None
    m = None if mult is None else torch.from_numpy(mult).to(device)
    b = None if bias is None else torch.from_numpy(bias).to(device)
    if budget_to is not None:
        bt = torch.from_numpy(np.ascontiguousarray(budget_to)).to(device)
        bf = None if budget_from is None else torch.from_numpy(np.ascontiguousarray(budget_from)).to(device)
        acc = psb.conv2d_progressive(q, x, bt, bf, stride=L.stride, pad=L.pad, seed=L.seed, layer_id=L.layer_id,
                                     acc=acc, y=y, mult=m, bias=b, shared=shared)
    elif L.linear:
        S = L.S if S is None else S
        x2 = x.reshape(n, -1)
        acc2 = torch.empty((n, oc), dtype=torch.int32, device=device)
        y2 = None if y is None else y.reshape(n, oc)
        psb.linear(q, x2, S, seed=L.seed, layer_id=L.layer_id, acc=acc2, y=y2, mult=m, bias=b, shared=shared)
        acc = acc2.reshape(n, oc, 1, 1)
    else:
        S = L.S if S is None else S
        acc = psb.conv2d(q, x, S, stride=L.stride, pad=L.pad, seed=L.seed, layer_id=L.layer_id, y=y, mult=m, bias=b,
                         shared=shared)
    torch.cuda.synchronize()
    return acc.cpu().numpy(), (None if y is None else y.cpu().numpy())


def pack_from_oracle(q):
    """The export format (sign<<31 | shift<<23 | mantissa, dead = 0x7F800000) from the oracle's arrays."""
    mant = np.rint(q.p * 2.0 ** 23).astype(np.uint32)
    word = (np.where(q.sign < 0, 1, 0).astype(np.uint32) << 31) | (q.shift.astype(np.uint32) << 23) | mant
    return np.where(q.sign == 0, np.uint32(0x7F800000), word).astype(np.uint32)
