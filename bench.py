#!/usr/bin/env python3
"""Benchmark of the sensitivity hot path on one MI355X.

A step is one pass of the whole device path over one decoder block's operand and gradient
tensors, already resident in HBM: per-tensor absmax + scales, then the fused two-format
sensitivity pass over the 7 linears and the 2 BGEMMs (amp_absmax_scale, amp_sens_block), each
call doing its own set-up (validation, work table, table to the device) as a calibration loop that
sees new buffers every time would.  Several distinct blocks (fresh seeds) stay resident and the steps
rotate over them, so no step finds its operands in a cache.  After the K steps (K = 32 is the
32-block sweep of the headline workload) the small statistics are copied to the host, the epilogue
of Sec. 2.2 builds the group tables from every step's own sums and amp_select_subgraphs solves
eq. (ip); that host tail is inside the timed region.

value = (bytes of x and xdot that the kernels of a step are defined to read from HBM) * K / wall
time of the timed region, in GB/s.  Per step that is 2 B per element of x for the absmax pass plus,
for the sensitivity pass, 4 B per (element, sample) pair, except that a weight shared by the
samples is read once per batch of 8 samples against their 8 gradients; masked causal entries,
partial sums and tables are not counted.  The same step priced at 4 B per pair for every sample
(as if W were re-read with each sample's gradient) is reported beside it.  "roofline" is the
longest fused sensitivity launch alone, timed with HIP events recorded by the library on the
launch stream.  "cpu_baseline" times the CPU oracle on a bounded sample of the same tensors.

Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np
import torch

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
METRIC = "sensitivity-pass HBM GB/s (bytes of x+ẋ read) and % of MI355X HBM peak"


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def build_workload(name, dev, block=0):
    from paper_2505_13060_amd import workloads as wl
    if name == "config2":
        return wl.config2_block(dev, block=block), "config2: 32-block Llama-7B-shaped sweep, one block (7 linears + QK^T + PV, S=2048, R=16, E4M3+E5M2) per step"
    if name == "config1":
        return wl.config1(dev, block=block), "config1: one Llama-7B-shaped block, S=2048, R=8, E4M3+E5M2"
    if name == "config3":
        return wl.config3(dev), "config3: 70B-shaped block, S=4096, R=8, GQA 64/8, E4M3"
    if name == "config4":
        return wl.config4(dev), "config4: 64 ragged expert linears + 24 BGEMMs at S=512, R=32, E4M3+E5M2"
    if name == "config0":
        return wl.config0(dev, seed_base=100 * block), "config0: one linear 1024x1024, R=4, E4M3"
    raise SystemExit("unknown workload " + name)


# ---- host tail: epilogue of Sec. 2.2 and the selection of eq. (ip) ------------------------------

def time_gains(workload, amp, delta=0.5):
    """Theoretical time gain per op (Sec. 2.3.2): MACs x the time saved per MAC; FP8 halves the MAC
    time.  A BGEMM's MAC count R*H*S*S*D is written in the paper's N*C^2 form with N = R*H*D, C = S."""
    g = {}
    for op in workload.linears:
        g[op.name] = amp.amp_time_gain_macs(0, int(op.row_offsets[-1]), op.C, op.K, delta)
    for op in workload.bgemms:
        H, S, D = op.x0.shape[1], op.x0.shape[2], op.x1.shape[3]
        g[op.name] = amp.amp_time_gain_macs(1, op.R * H * D, S, S, delta)
    return g


def host_tail(workloads, results, n_steps, amp):
    """Per-layer loss MSE from every step's own measured sums (step k ran on block k mod B), group
    tables for the Llama block partition of the paper's Appendix B figure ({q,k,v,qk,av}, {o},
    {gate,up}, {down}), then eq. (ip) over all steps' groups under a budget of 1e-3 x the loss MSE of
    the most aggressive configuration."""
    per_block = []
    for workload, res in zip(workloads, results):
        fmts = workload.fmts
        nf = len(fmts)
        layer = {}
        for k, op in enumerate(workload.linears):
            layer[op.name] = amp.amp_layer_loss_mse(res["linear"][k], fmts)
        for k, op in enumerate(workload.bgemms):
            layer[op.name] = amp.amp_layer_loss_mse(res["bgemm"][k], fmts)
        gains = time_gains(workload, amp)
        names = list(layer)
        attn = [n for n in names if n in ("q_proj", "k_proj", "v_proj", "qk_matmul", "av_matmul")]
        if len(attn) == 5:
            groups = [attn, ["o_proj"], ["gate_proj", "up_proj"], ["down_proj"]]
        else:
            groups = [[n] for n in names]           # J = L special case
        tables = []
        for g in groups:
            lm = np.zeros((len(g), nf + 1))
            lg = np.zeros((len(g), nf + 1))
            for i, n in enumerate(g):
                lm[i, 1:] = layer[n][2]                               # measured first-order loss MSE
                lg[i, 1:] = gains[n]
            tables.append(amp.amp_group_tables(lm, lg))
        per_block.append(tables)
    n_choices, gains_all, mses = [], [], []
    for k in range(n_steps):
        for d, c in per_block[k % len(per_block)]:
            n_choices.append(d.size)
            mses.append(d)
            gains_all.append(c)
    total = sum(float(m.max()) for m in mses)
    budget = 1e-3 * total
    t0 = time.perf_counter()
    choice, tg, td = amp.amp_select_subgraphs(np.array(n_choices, dtype=np.int32), np.concatenate(gains_all),
                                              np.concatenate(mses), budget)
    t1 = time.perf_counter()
    return dict(groups=len(n_choices), budget=budget, total_gain=tg, total_mse=td,
                quantised_groups=int(np.count_nonzero(choice)), solve_ms=(t1 - t0) * 1e3,
                tables="every step's own sums (step k on resident block k mod %d); gain = MACs x 0.5 "
                       "(amp_time_gain_macs)" % len(per_block))


# ---- CPU baseline: the oracle on a bounded sample --------------------------------------------

def cpu_baseline(workload, target_seconds=15.0):
    """The oracle's per-tensor routine on a bounded sample (the per-row routine does the same
    arithmetic per element; the baseline is quoted for the headline mode)."""
    import oracle
    from paper_2505_13060_amd.workloads import to_bits
    threads = max(1, min(16, os.cpu_count() or 1))
    per_thread_rate = 20e6                                      # pair-formats per second, rough
    budget = per_thread_rate * threads * target_seconds
    nf = len(workload.fmts)
    tasks, picked, used = [], [], 0.0
    for op in workload.linears:
        if used >= budget:
            break
        x, dx, w, dw = to_bits(op.x), to_bits(op.dx), to_bits(op.w), to_bits(op.dw)
        scx = [oracle.absmax_scale(x.reshape(-1), f) for f in workload.fmts]
        scw = [oracle.absmax_scale(w.reshape(-1), f) for f in workload.fmts]
        took = 0
        for r in range(op.R):
            if used >= budget:
                break
            a, b = int(op.row_offsets[r]) * op.C, int(op.row_offsets[r + 1]) * op.C
            for fi, f in enumerate(workload.fmts):
                tasks.append((x.reshape(-1)[a:b], dx.reshape(-1)[a:b], b - a, scx[fi][1], scx[fi][2], f))
                tasks.append((w.reshape(-1), dw[r].reshape(-1), op.K * op.C, scw[fi][1], scw[fi][2], f))
            used += nf * ((b - a) + op.K * op.C)
            took += 1
        picked.append("%s samples 0..%d" % (op.name, took - 1))
    pairs = sum(t[2] for t in tasks) / nf

    def run(t):
        return oracle.sens_operand(t[0], t[1], 1, t[2], t[3], t[4], t[5])

    t0 = time.perf_counter()
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(run, tasks))
    dt = time.perf_counter() - t0
    return {"value": pairs * 4 / dt / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "seconds": dt,
            "sample": "X and W operands (all %d formats) of %s: %.1f M pairs; scales precomputed, "
                      "device-to-host copy not timed" % (nf, "; ".join(picked), pairs / 1e6)}


def kernel_source_sha():
    """Hash of the sources the kernels are built from; a counter summary under profiles/ names the
    hash it was measured at."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2505_13060_amd", "csrc")
    for name in ("kernels.hip", "walk.h", "internal.h"):
        h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(kernel_label, workload_name):
    """HBM bytes per launch of the named kernel from the committed rocprofv3 counter summaries
    (FETCH_SIZE and WRITE_SIZE runs of this same command, scaled by a plain copy of known size).
    None if no summary under profiles/ covers the kernel on this workload, or if the summary was
    measured on other kernel sources than the ones in this tree (line "kernel_source_sha = ...")."""
    kernel = (kernel_label or "").split(" ")[0].rstrip(",")
    tag = "traffic_bytes_per_launch(%s, %s) =" % (kernel, workload_name)
    folder = os.path.join(ROOT, "profiles")
    try:
        names = sorted(os.listdir(folder))
    except OSError:
        return None
    for name in names:
        if not name.endswith(".md"):
            continue
        try:
            lines = open(os.path.join(folder, name)).read().splitlines()
        except OSError:
            continue
        sha = [ln.split("=")[1].strip() for ln in lines if ln.startswith("kernel_source_sha =")]
        for line in lines:
            if line.startswith(tag):
                return float(line.split("=")[1]) if sha and sha[0] == kernel_source_sha() else None
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=32)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="config2")
    ap.add_argument("--blocks", type=int, default=0,
                    help="distinct resident blocks the steps rotate over (0 = 4 for config2 at 28 GB each, 16 "
                         "for config0 so that a rotation exceeds the 256 MB cache, 1 otherwise)")
    ap.add_argument("--calls", choices=["oneshot", "plan"], default="oneshot",
                    help="oneshot: every step's calls do their own set-up (headline); plan: set-up once per "
                         "block outside the timed region, steps replay the plans with amp_run")
    ap.add_argument("--scales", choices=["tensor", "rows", "rows-single-read"], default="tensor",
                    help="scale granularity: one per tensor (headline) or one per row (per token / per "
                         "output channel / per row of a BGEMM operand); rows-single-read: the sensitivity "
                         "pass computes the row scales of the activations and BGEMM operands itself, "
                         "every row is fetched once")
    ap.add_argument("--scale-block", type=int, default=0,
                    help="with --scales rows / rows-single-read: one scale per 1 x N block of every dense row "
                         "(N must divide the row lengths, e.g. 128) instead of one per row; causal rows keep one each")
    ap.add_argument("--scale-rule", choices=["amax", "pow2"], default="amax",
                    help="amax: scale = amax / FMAX (headline); pow2: the smallest power of two that is large "
                         "enough (AMP_SCALE_POW2 on both calls: the sensitivity kernels then cast with gfx950's "
                         "scaled FP8 conversions)")
    ap.add_argument("--settle", type=float, default=6.0,
                    help="seconds to leave the GPU idle between generating the inputs and the warm-up: for a "
                         "few seconds after a process has freed tens of GB of device memory every kernel on "
                         "the device streams about 3 %% slower")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference reading for HBM counters)")
    args = ap.parse_args()
    if args.scale_block and args.scales == "tensor":
        print("bench.py: --scale-block needs --scales rows or rows-single-read", file=sys.stderr)
        sys.exit(2)
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); multi-GPU runs are not part of it",
              file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        sys.exit(3)

    import paper_2505_13060_amd as amp
    from paper_2505_13060_amd.pipeline import RowSensPass, SensPass
    dev = "cuda:0"
    torch.cuda.set_device(0)
    n_blocks = args.blocks or {"config2": 4, "config0": 16}.get(args.workload, 1)
    n_blocks = max(1, min(n_blocks, args.steps))
    log("generating %d block(s) of %s on %s" % (n_blocks, args.workload, torch.cuda.get_device_name(0)))
    t0 = time.perf_counter()
    workloads, passes = [], []
    rule = amp.SCALE_POW2 if args.scale_rule == "pow2" else 0
    for b in range(n_blocks):
        workload, label = build_workload(args.workload, dev, block=b)
        workloads.append(workload)
        # linears and BGEMMs of the block in one call: one table, one set-up, one streaming launch
        plan = args.calls == "plan"
        passes.append(SensPass(workload, dev, one_call=True, plan=plan, rule=rule) if args.scales == "tensor"
                      else RowSensPass(workload, dev, one_call=True, plan=plan, rule=rule, block=args.scale_block,
                                       single_read=args.scales == "rows-single-read"))
    torch.cuda.synchronize()
    workload = workloads[0]
    pairs = workload.pairs()
    log("%.1f M pairs per step (%.2f GB), generated in %.1f s" % (pairs / 1e6, pairs * 4 / 1e9, time.perf_counter() - t0))
    if args.scales != "tensor":
        label += ("; one scale per 1 x %d block of a row" % args.scale_block if args.scale_block else "; one scale per row") + \
                 (", computed by the sensitivity pass (single read)" if args.scales != "rows" else "")
    if rule:
        label += "; power-of-two scales, cast by the scaled FP8 conversions"
    label += "; steps rotate over %d distinct resident block(s)" % n_blocks
    # elements the absmax passes of a step read: every operand once, except those whose row scales
    # the sensitivity pass computes itself
    abs_elems = 0
    for op in workload.linears:
        abs_elems += op.K * op.C + (0 if args.scales == "rows-single-read" else int(op.row_offsets[-1]) * op.C)
    for op in workload.bgemms:
        abs_elems += 0 if args.scales == "rows-single-read" else op.pairs()

    if args.calibrate_copy:
        src = torch.ones(1 << 28, device=dev, dtype=torch.float32)       # 1 GiB
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.settle > 0:
        torch.cuda.synchronize()
        time.sleep(args.settle)

    def results():
        return [p.results(scales=False) for p in passes]

    for k in range(args.warmup):
        passes[k % n_blocks].run()
    # the warm-up ends like the timed region does: read-back, epilogue, selection (the first
    # device-to-host copy of a process sets up the runtime's staging)
    host_tail(workloads, results(), args.steps, amp)
    torch.cuda.synchronize()
    # launches of the fused kernels per step (the weight kernel, then the streaming kernel for the
    # activations and the BGEMM operands; with row scales one streaming launch per class of rows)
    amp.amp_profile_enable(16)
    passes[0].run()
    launches_per_step = len(amp.amp_profile_read(16)[0])
    amp.amp_profile_enable(args.steps * launches_per_step)

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        passes[k % n_blocks].run()
    t_enq = time.perf_counter()
    torch.cuda.synchronize()
    t_dev = time.perf_counter()
    res = results()                                                        # copies the sums
    tail = host_tail(workloads, res, args.steps, amp)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    log("enqueue %.2f ms, device done after %.2f ms, read-back + epilogue + selection %.2f ms" %
        ((t_enq - t0) * 1e3, (t_dev - t0) * 1e3, (t1 - t_dev) * 1e3))

    kinds = amp.amp_profile_kinds(args.steps * launches_per_step)
    ms, lp, lb = amp.amp_profile_read(args.steps * launches_per_step)
    amp.amp_profile_enable(0)
    wall = t1 - t0
    if launches_per_step <= 0 or len(ms) != args.steps * launches_per_step:
        raise SystemExit("bench.py: the library reported %d launch records for %d steps x %d launches"
                         % (len(ms), args.steps, launches_per_step))
    sens_bytes_step = float(lb.reshape(args.steps, launches_per_step)[0].astype(np.float64).sum())
    abs_bytes_step = abs_elems * 2.0
    bytes_step = sens_bytes_step + abs_bytes_step
    value = bytes_step * args.steps / wall / 1e9
    log("device steps + host tail: %.3f s over %d steps" % (wall, args.steps))
    kernel_of = {
        amp.KERNEL_WEIGHTS: "sens_w_kernel (weights of the linears)",
        amp.KERNEL_WEIGHTS + 1: "sens_w_kernel, per-channel scales (weights of the linears)",
        amp.KERNEL_STREAM: "sens_kernel (activations of the linears and BGEMM operands)",
        amp.KERNEL_STREAM + 1: "sens_wrows_kernel (one scale per row: long and causal rows)",
        amp.KERNEL_STREAM + 2: "sens_rows_kernel (one scale per row: other row shapes)",
        amp.KERNEL_STREAM + 3: "sens_wrows_kernel, short-row variant (one scale per row: rows of a power-of-two length below 512)",
        amp.KERNEL_STREAM + 4: "sens_fused_rows_kernel (absmax, scales and sums in one read; rows held in registers)",
        amp.KERNEL_STREAM + 5: "sens_fused_rows_kernel, rows staged in LDS (up to 32 KiB per workgroup)",
        amp.KERNEL_STREAM + 6: "sens_fused_rows_kernel, rows staged in LDS (up to 48 KiB per workgroup)",
    }
    names = [kernel_of.get(int(k), "launch of kind %d" % k) for k in kinds[:launches_per_step]]
    launch_detail = []
    per_ms = ms.reshape(args.steps, launches_per_step).mean(axis=0)
    per_min = ms.reshape(args.steps, launches_per_step).min(axis=0)
    per_pairs = lp.reshape(args.steps, launches_per_step)[0].astype(np.float64)
    per_bytes = lb.reshape(args.steps, launches_per_step)[0].astype(np.float64)
    for name, t, tmin, n, nb in zip(names, per_ms, per_min, per_pairs, per_bytes):
        log("  %-42s %.3f ms (min %.3f)  %8.1f M pairs  reads %.2f GB: %.0f GB/s  (%.0f GB/s at 4 B per pair)" %
            (name, t, tmin, n / 1e6, nb / 1e9, nb / t / 1e6, n * 4 / t / 1e6))
        launch_detail.append({"kernel": name, "ms": float(t), "ms_min": float(tmin), "pairs": n, "bytes": nb,
                              "GB/s": nb / float(t) / 1e6, "GB/s_at_4B_per_pair": n * 4.0 / float(t) / 1e6})
    # the dominant kernel: the launch that takes longest
    dom = max(launch_detail, key=lambda d: d["ms"])
    kern_bytes = dom["bytes"] if dom else float("nan")
    kern_ms = dom["ms"] if dom else float("nan")
    achieved = dom["GB/s"] if dom else float("nan")
    all_ms = float(sum(d["ms"] for d in launch_detail))
    all_bytes = float(sum(d["bytes"] for d in launch_detail))
    all_gbs = all_bytes / all_ms / 1e6 if launch_detail else float("nan")

    # absmax alone (secondary line)
    torch.cuda.synchronize()
    ta = time.perf_counter()
    for k in range(args.steps):
        passes[k % n_blocks].absmax()
    torch.cuda.synchronize()
    abs_ms = (time.perf_counter() - ta) / args.steps * 1e3

    # the same steps with the set-up of every call kept (plans): what a calibration loop that revisits
    # its buffers pays, and what the set-up costs (secondary line; the headline does the set-up per step)
    other = None
    if args.calls == "oneshot" and args.scales == "tensor":
        plans = [SensPass(w, dev, plan=True, rule=rule) for w in workloads]
        for k in range(min(args.warmup, 2 * n_blocks)):
            plans[k % n_blocks].run()
        torch.cuda.synchronize()
        tp0 = time.perf_counter()
        for k in range(args.steps):
            plans[k % n_blocks].run()
        tp_enq = time.perf_counter()
        torch.cuda.synchronize()
        tp1 = time.perf_counter()
        other = {"ms_per_step": (tp1 - tp0) / args.steps * 1e3, "host_enqueue_ms_per_step": (tp_enq - tp0) / args.steps * 1e3,
                 "GB/s": bytes_step * args.steps / (tp1 - tp0) / 1e9,
                 "note": "amp_run of plans set up once per block (no host tail in this figure)"}
        log("plans: %.3f ms per step, host %.3f ms per step" % (other["ms_per_step"], other["host_enqueue_ms_per_step"]))

    out = {
        "metric": METRIC, "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": wall / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": label, "pairs_per_step": pairs, "bytes_per_step": bytes_step,
                   "bytes_per_step_absmax": abs_bytes_step, "bytes_per_step_sens": sens_bytes_step,
                   "formats": ["E4M3" if f == 0 else "E5M2" for f in workload.fmts],
                   "resident_blocks": n_blocks, "calls": args.calls, "scale_rule": args.scale_rule,
                   "weights": "resident mode: all R weight gradients of an op are in HBM, W is read "
                              "once per batch of 8 samples; activations and BGEMM operands 4 B per pair"},
        "pct_of_hbm_peak": 100.0 * value / HBM_PEAK_GBS,
        "value_at_4B_per_pair": pairs * 4.0 * args.steps / wall / 1e9,
        "roofline": {"bound": "hbm", "kernel": dom["kernel"] if dom else None,
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(dom["kernel"] if dom else None, args.workload),
                     "bytes_per_launch": kern_bytes, "ms_per_launch": kern_ms,
                     "ms_per_launch_min": dom["ms_min"] if dom else None,
                     "bytes": "operand bytes the kernel is defined to read: 4 B per (element, sample) pair, "
                              "except that the weight kernel reads W once per batch of 8 samples",
                     "all_fused_launches": {"ms_per_step": all_ms, "bytes_per_step": all_bytes, "GB/s": all_gbs,
                                            "frac": all_gbs / HBM_PEAK_GBS,
                                            "GB/s_at_4B_per_pair": pairs * 4.0 / all_ms / 1e6},
                     "launches_per_step": launch_detail},
        "absmax": {"ms_per_step": abs_ms, "GB/s": abs_bytes_step / (abs_ms * 1e-3) / 1e9,
                   "bytes_per_step": abs_bytes_step},
        "select": tail,
        "timed_region": {"device_ms": (t_dev - t0) * 1e3, "host_enqueue_ms": (t_enq - t0) * 1e3,
                         "host_tail_ms": (t1 - t_dev) * 1e3, "idle_before_warmup_s": args.settle},
    }
    if other is not None:
        out["plans"] = other
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample")
        out["cpu_baseline"] = cpu_baseline(workload, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
