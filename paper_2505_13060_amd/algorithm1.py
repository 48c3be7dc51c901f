"""The paper's top-level procedure (Algorithm 1, App. A) assembled from the library's calls:

  1. partition the model into sequential sub-graphs     amp_partition_sequential (App. B), or given
  2. sensitivity calibration                            capture.py -> amp_absmax_scale / amp_sens_*
  3. gain of every group and configuration              theoretical MAC or memory gain (Sec. 2.3.2,
                                                        2.3.3); measured times may be passed instead
  4. solve eq. (ip) under the budget tau^2 E[g^2]       amp_select_subgraphs

Marshalling and bookkeeping only: every number (sums, loss MSE, tables, selection) is produced by
libampsens.  The empirical time gain of Sec. 2.3.1 needs the target accelerator and is an input
here (`gains`), not something this module measures.
"""
from collections import OrderedDict

import numpy as np

from . import (amp_group_tables, amp_layer_loss_mse, amp_memory_gain, amp_mse_budget, amp_partition_sequential,
               amp_select_ordered, amp_select_subgraphs, amp_time_gain_macs)


def layer_loss_mse(sums, fmts, statistic="measured"):
    """{op: loss MSE per candidate format [n_fmts]} from the library's sums {op: [R, n_fmts, 4]}.
    statistic: "measured" = mean_r (E_0 + E_1), the first-order term with the actual rounding
    error; "model" = s_l * alpha_f, the uniform-noise model of Sec. 2.2."""
    out = OrderedDict()
    for name, s in sums.items():
        s_layer, d_model, d_meas = amp_layer_loss_mse(s, fmts)
        out[name] = d_meas if statistic == "measured" else d_model
    return out


def theoretical_gains(ops, n_fmts, objective="time", delta=0.5):
    """{op: gain per candidate format [n_fmts]} from shapes.  ops: {name: dict(kind="linear",
    N=tokens, C=..., K=...) or dict(kind="bgemm", N=rows, C=..., K=...)}.  objective "time": the MAC
    count times delta (Sec. 2.3.2; delta = time saved per MAC relative to BF16, the same for every
    FP8 format); "memory": C*K*delta for a linear layer's weight, 0 for a BGEMM (Sec. 2.3.3)."""
    out = OrderedDict()
    for name, o in ops.items():
        bg = 1 if o["kind"] == "bgemm" else 0
        if objective == "time":
            g = amp_time_gain_macs(bg, o["N"], o["C"], o.get("K", o["C"]), delta)
        else:
            g = amp_memory_gain(bg, o["C"], o.get("K", o["C"]), delta)
        out[name] = np.full(n_fmts, g)
    return out


def partition(op_names, edges, quantizable=None):
    """Groups (lists of op names, in execution order) of the DAG whose vertices are op_names and
    whose edges are (src name, dst name) pairs; quantizable: names of the linear operations
    (default: all).  Add a virtual source / sink yourself if the graph has several."""
    index = {n: i for i, n in enumerate(op_names)}
    q = None if quantizable is None else [1 if n in set(quantizable) else 0 for n in op_names]
    group_of, n_groups = amp_partition_sequential(len(op_names), [(index[a], index[b]) for a, b in edges], q)
    groups = [[] for _ in range(n_groups)]
    for n, g in zip(op_names, group_of):
        if g >= 0:
            groups[g].append(n)
    return groups


def build_tables(groups, mse, gains):
    """Concatenated tables of eq. (ip): per group the F^L_j columns of Q_j with choice 0 = every
    layer at high precision (loss MSE 0, gain 0).  Returns (n_choices, gain, mse) arrays."""
    n_choices, G, D = [], [], []
    for g in groups:
        nf = len(mse[g[0]])
        lm = np.zeros((len(g), nf + 1))
        lg = np.zeros((len(g), nf + 1))
        for i, n in enumerate(g):
            lm[i, 1:] = mse[n]
            lg[i, 1:] = gains[n]
        d, c = amp_group_tables(lm, lg)
        n_choices.append(d.size)
        D.append(d)
        G.append(c)
    return np.array(n_choices, dtype=np.int32), np.concatenate(G), np.concatenate(D)


def decode(groups, choice, fmts):
    """{op: format, or None for high precision} from the chosen column of every group (column p
    is the base-(F+1) digit string of p, first layer of the group least significant)."""
    F = len(fmts) + 1
    out = OrderedDict()
    for g, p in zip(groups, choice):
        for i, n in enumerate(g):
            digit = (int(p) // F ** i) % F
            out[n] = None if digit == 0 else fmts[digit - 1]
    return out


def select(sums, mean_g2, tau, groups, gains, fmts, statistic="measured", strategy="ip", order=None):
    """Step 4: the mixed-precision configuration under the loss-MSE budget tau^2 E[g^2] (eq. (ip)).
    strategy "ip" solves the integer program; "prefix" / "ordered" walk the groups in (the given)
    order as the baselines of Sec. 3.1 do.  Returns (config {op: format or None}, info)."""
    mse = layer_loss_mse(sums, fmts, statistic)
    n_choices, G, D = build_tables(groups, mse, gains)
    budget = amp_mse_budget(tau, mean_g2)
    if strategy == "ip":
        choice, total_gain, total_mse = amp_select_subgraphs(n_choices, G, D, budget)
    else:
        choice, total_gain, total_mse = amp_select_ordered(n_choices, G, D, budget, order)
    return decode(groups, choice, fmts), dict(budget=budget, total_gain=total_gain, total_mse=total_mse,
                                              choice=np.asarray(choice))


def tradeoff_curve(sums, mean_g2, taus, groups, gains, fmts, statistic="measured", strategy="ip", order=None):
    """Gain and predicted loss MSE over a grid of thresholds (the shape of the paper's
    accuracy-versus-gain figures, on whatever statistics were measured)."""
    mse = layer_loss_mse(sums, fmts, statistic)
    n_choices, G, D = build_tables(groups, mse, gains)
    rows = []
    for tau in taus:
        budget = amp_mse_budget(tau, mean_g2)
        if strategy == "ip":
            _, tg, td = amp_select_subgraphs(n_choices, G, D, budget)
        else:
            _, tg, td = amp_select_ordered(n_choices, G, D, budget, order)
        rows.append((float(tau), tg, td))
    return rows


def calibrate(model, samples, loss_fn, fmts, device, resident=True, bgemm_setter=None):
    """Step 2 on a PyTorch model: one forward/backward pass per sample through the capture layer.
    loss_fn(model, sample) returns the scalar loss; bgemm_setter(cap.bgemm) lets the model route its
    attention matmuls through the capture.  Returns (sums, E[g^2], ops) with ops the shapes
    theoretical_gains needs."""
    from . import capture as cp
    sink = cp.ResidentSink(fmts, device) if resident else cp.StreamSink(fmts, device)
    shapes = OrderedDict()

    class Tee:
        def add_sample(self, recs, loss):
            for r in recs:
                if r.name in shapes:
                    continue
                if r.kind == "linear":
                    K, C_ = r.w.shape
                    shapes[r.name] = dict(kind="linear", N=r.x.numel() // C_, C=C_, K=K)
                else:                                            # [.., M, K] x [.., K, N]
                    shapes[r.name] = dict(kind="bgemm", N=r.x.numel() // r.x.shape[-1], C=r.x.shape[-1],
                                          K=r.x1.shape[-1])
            sink.add_sample(recs, loss)

    cap = cp.Capture(model, Tee())
    if bgemm_setter is not None:
        bgemm_setter(cap.bgemm)
    try:
        for s in samples:
            cap.sample(lambda: loss_fn(model, s))
    finally:
        cap.close()
        if bgemm_setter is not None:
            import torch
            bgemm_setter(lambda name, a, b, causal_a=False: torch.matmul(a, b))
    sums, mean_g2 = sink.finalize()
    return sums, mean_g2, shapes
