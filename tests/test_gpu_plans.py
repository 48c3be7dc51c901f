"""Plans (set-up once, amp_run many times) and HIP graph capture of the library's calls.

A run must read the operands and scales as they are when it executes: the inputs are changed
between runs and every run is compared with the oracle.  Captured graphs (one-shot calls, whose
descriptor tables travel as kernel arguments, and plan runs) are replayed several times with eager
work and synchronisations in between, and every replay must reproduce the eager result bit for bit."""
import sys

import numpy as np
import pytest
import torch

import paper_2505_13060_amd as amp
from paper_2505_13060_amd import workloads as wl
from paper_2505_13060_amd.pipeline import RowSensPass, SensPass
import parity

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def say(msg):
    print("[gpu-test] " + msg, flush=True)
    sys.stdout.flush()


def to_device(workload):
    for op in workload.linears:
        op.x, op.dx, op.w, op.dw = (t.to(DEV) for t in (op.x, op.dx, op.w, op.dw))
    for op in workload.bgemms:
        op.x0, op.dx0, op.x1, op.dx1 = (t.to(DEV) for t in (op.x0, op.dx0, op.x1, op.dx1))
    return workload


def small_block():
    return to_device(wl.config1("cpu", R=3, S=136, hidden=256, ffn=520, H=2, D=64))


def ragged():
    return to_device(wl.config4("cpu", R=5, experts=6, C=512, K=176, tok_lo=1, tok_hi=40, n_bgemm=4, S=72, H=2, D=32))


def snapshot(p):
    r = p.results()
    return [a.copy() for a in r["linear"] + r["bgemm"]] + [r["scale"].copy(), r["inv"].copy(), r["amax"].copy()]


def same_bits(a, b):
    return all(np.array_equal(parity.bits32(x), parity.bits32(y)) for x, y in zip(a, b))


def perturb(workload, k):
    """Changes operands in place (same buffers, so plans and graphs stay valid): new amax, new sums."""
    for op in workload.linears:
        op.x.mul_(1.5 if k % 2 else 0.5)
        op.w[0, :8] = float(3 + k)
    for op in workload.bgemms:
        op.x1.mul_(-2.0)
        op.dx0.mul_(0.5)


@pytest.mark.parametrize("make", [small_block, ragged])
def test_plan_runs_follow_the_inputs(make):
    w = make()
    say("plan: set-up once, three runs on changing inputs (%s)" % w.name)
    p = SensPass(w, DEV, plan=True)
    for k in range(3):
        p.d_out.fill_(-1.0)
        p.run()
        parity.check_workload(w, p.results())
        one = SensPass(w, DEV, one_call=True)
        one.run()
        assert same_bits(snapshot(p), snapshot(one))
        perturb(w, k)


def test_plan_runs_with_row_scales():
    w = small_block()
    say("plan with one scale per row: two runs on changing inputs")
    p = RowSensPass(w, DEV, plan=True)
    for k in range(2):
        p.run()
        parity.check_workload_rows(w, p.results())
        perturb(w, k)


@pytest.mark.parametrize("mode", ["oneshot", "plan"])
@pytest.mark.parametrize("make", [lambda: to_device(wl.config0("cpu")), ragged, small_block])
def test_graph_replays_match_eager(make, mode):
    w = make()
    say("HIP graph of one step (%s, %s calls): capture, 4 replays with eager work in between" % (w.name, mode))
    p = SensPass(w, DEV, one_call=True, plan=(mode == "plan"))
    p.run()                                                 # warm-up: occupancy queries, module load
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=stream):
        p.run()                                             # enqueues on the capturing (current) stream
    torch.cuda.synchronize()
    for k in range(4):
        # eager reference on the current inputs
        p.d_out.zero_()
        p.run()
        want = snapshot(p)
        parity.check_workload(w, p.results())
        # destroy the outputs, do unrelated eager work, then replay
        p.d_out.fill_(float("nan"))
        p.d_scale.zero_()
        p.d_inv.zero_()
        junk = torch.randn(1 << 20, device=DEV).sum().item()
        assert np.isfinite(junk)
        graph.replay()
        torch.cuda.synchronize()
        got = snapshot(p)
        assert same_bits(got, want), "replay %d differs from the eager pass" % k
        perturb(w, k)
