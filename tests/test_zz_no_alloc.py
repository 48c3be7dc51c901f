"""amp_sens_block_static: the sensitivity pass with the library's own fixed device array as its
workspace, for callers that cannot allocate.  Its sums must be those of amp_sens_block bit for bit
(same kernels, same chunking), on two calls in a row of which the second is smaller (the array keeps
the first call's contents), and a call that does not fit must be refused before any launch."""
import sys

import numpy as np
import pytest
import torch

import paper_2505_13060_amd as amp
from paper_2505_13060_amd import workloads as wl
from paper_2505_13060_amd.pipeline import SensPass
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


def test_static_workspace_matches_the_workspace_call_twice_in_a_row():
    big = to_device(wl.config1("cpu", R=3, S=264, hidden=512, ffn=1032, H=4, D=64))
    small = to_device(wl.config4("cpu", R=2, experts=3, C=256, K=88, tok_lo=1, tok_hi=24, n_bgemm=2, S=40, H=2, D=32))
    for w in (big, small):                                  # the second call is the smaller one
        p = SensPass(w, DEV, one_call=True)
        p.absmax()
        assert p.ws_block.numel() <= amp.STATIC_WORKSPACE_BYTES
        say("amp_sens_block on %s (workspace %d bytes), then amp_sens_block_static" % (w.name, p.ws_block.numel()))
        p.sens()
        want = p.d_out.clone()
        torch.cuda.synchronize()
        parity.check_workload(w, p.results())
        p.d_out.fill_(float("nan"))
        amp.amp_sens_block_static(p.lin_desc, p.bg_desc, p.fmts, p.d_out)
        torch.cuda.synchronize()
        got = p.d_out
        assert torch.equal(got.view(torch.int32), want.view(torch.int32)), w.name
    # once more on the larger one: nothing of the smaller call's contents may matter
    p = SensPass(big, DEV, one_call=True)
    p.run()
    want = p.d_out.clone()
    p.d_out.zero_()
    amp.amp_sens_block_static(p.lin_desc, p.bg_desc, p.fmts, p.d_out)
    torch.cuda.synchronize()
    assert torch.equal(p.d_out.view(torch.int32), want.view(torch.int32))


def test_static_workspace_refuses_what_does_not_fit():
    # one dense operand of 2^31 elements would need a chunk map and partials of 4 MiB ... 32 MiB:
    # nothing is dereferenced, the call must answer on the host
    n = 1 << 33
    d = amp.BgemmDesc()
    d.x0 = d.dx0 = d.x1 = d.dx1 = 4096
    d.layout0, d.layout1, d.R = amp.dense(n), amp.dense(0), 1
    d.scale0 = d.inv0 = d.scale1 = d.inv1 = 4096
    assert amp.amp_sens_bgemm_workspace_bytes([d], 2) > amp.STATIC_WORKSPACE_BYTES
    out = torch.zeros(1, 2, 4, device=DEV)
    with pytest.raises(amp.AmpError) as ei:
        amp.amp_sens_block_static([], [d], [amp.E4M3, amp.E5M2], out)
    assert ei.value.status == amp.ERR_WORKSPACE_TOO_SMALL
    # an empty call is fine and launches nothing
    amp.amp_sens_block_static([], [], [amp.E4M3], out)
