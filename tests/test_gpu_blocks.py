"""One scale per 1 x B block of a row (AMP_ROWS_BLOCK): the tables amp_absmax_scale_rows writes for the
buffers described with rows of B elements must equal the oracle's block routine bit for bit, and the sums
of the sensitivity pass, told about the blocks through scale_rows (linears) or through the row length of a
dense layout (BGEMM operands), must match the oracle's sums for the same blocks: through the weight
kernel, the streaming kernels and the single-read pass."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2505_13060_amd as amp
from paper_2505_13060_amd import workloads as wl
from paper_2505_13060_amd.pipeline import RowSensPass
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


@pytest.mark.parametrize("block", [128, 64, 16])
@pytest.mark.parametrize("mode", ["two_pass", "single_read", "plan_stream_weights"])
def test_block_scales_on_a_reduced_block(block, mode):
    """Linears with 1 x B blocks on X and W, attention operands with blocks along their last dimension
    (the causal P keeps one scale per row); B = 128, 64 and 16 land in different kernels."""
    w = to_device(wl.config1("cpu", R=3, S=128, hidden=256, ffn=512, H=2, D=128))
    say("block scales %d, %s: %s, %.1f M pairs" % (block, mode, w.name, w.pairs() / 1e6))
    kw = dict(two_pass={}, single_read=dict(single_read=True),
              plan_stream_weights=dict(plan=True, flags=amp.PLAN_STREAM_WEIGHTS))[mode]
    p = RowSensPass(w, DEV, block=block, **kw)
    p.r_scale.fill_(float("nan"))
    p.r_inv.fill_(float("nan"))
    p.run()
    res = p.results()
    parity.check_workload_blocks(w, res, block)


def test_ragged_experts_with_block_scales():
    w = to_device(wl.config4("cpu", R=4, experts=5, C=512, K=176, tok_lo=1, tok_hi=40, n_bgemm=2, S=64, H=2, D=64))
    say("block scales 64 on ragged experts: %.1f M pairs" % (w.pairs() / 1e6))
    for kw in (dict(one_call=True), dict(single_read=True, one_call=True)):
        p = RowSensPass(w, DEV, block=64, **kw)
        p.run()
        parity.check_workload_blocks(w, p.results(), 64)


def test_block_flag_on_a_bgemm_descriptor_equals_the_shorter_row_length():
    """AMP_ROWS_BLOCK on a BGEMM descriptor with dense operands is the same call as giving the operands'
    layouts the block as their row length; a block that does not divide the row, a block without any
    row-scaled operand, and a causal operand with blocks are refused."""
    rng = np.random.default_rng(5)
    R, rows, cols, B = 2, 24, 256, 64
    n = rows * cols
    x = torch.from_numpy(rng.standard_normal(R * n).astype(np.float32)).to(torch.bfloat16).to(DEV)
    g = torch.from_numpy((rng.standard_normal(R * n) * 1e-2).astype(np.float32)).to(torch.bfloat16).to(DEV)
    n_blocks = R * n // B
    am = torch.zeros(n_blocks, device=DEV)
    ts = torch.zeros(n_blocks, 2, device=DEV)
    ti = torch.zeros(n_blocks, 2, device=DEV)
    fl = torch.zeros(1, dtype=torch.int32, device=DEV)
    fmts = [amp.E4M3, amp.E5M2]
    t = [amp.tensor(x, amp.dense(n, B), R)]
    wsb, nr = amp.amp_absmax_rows_workspace_bytes(t)
    assert nr == n_blocks
    wsa = torch.empty(max(wsb, 256), dtype=torch.uint8, device=DEV)
    amp.amp_absmax_scale_rows(t, fmts, am, ts, ti, fl, wsa)
    outs = []
    for lay, flag in ((amp.dense(n, cols), amp.ROWS_OPERAND0 | amp.rows_block(B)), (amp.dense(n, B), amp.ROWS_OPERAND0)):
        d = amp.bgemm_desc(x, g, lay, None, None, amp.dense(0), R, ts, ti, None, None, scale_rows=flag)
        out = torch.zeros(R, 2, 4, device=DEV)
        ws = torch.empty(amp.amp_sens_bgemm_workspace_bytes([d], 2), dtype=torch.uint8, device=DEV)
        amp.amp_sens_bgemm([d], fmts, out, ws)
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy())
    assert np.array_equal(parity.bits32(outs[0]), parity.bits32(outs[1]))
    xb = x.view(torch.int16).cpu().numpy().view(np.uint16)
    gb = g.view(torch.int16).cpu().numpy().view(np.uint16)
    for fi, f in enumerate(fmts):
        a_, sc, iv, _ = oracle.absmax_scale_blocks(xb, R * rows, cols, B, f)
        assert np.array_equal(parity.bits32(ts[:, fi].cpu().numpy()), parity.bits32(sc.reshape(-1)))
        for r in range(R):
            E, A = oracle.sens_operand_blocks(xb[r * n:(r + 1) * n], gb[r * n:(r + 1) * n], rows, cols, B,
                                              sc[r * rows:(r + 1) * rows], iv[r * rows:(r + 1) * rows], f)
            parity.assert_sum_close(outs[0][r, fi, 1], A, 0.0, "A")
            parity.assert_sum_close(outs[0][r, fi, 0], E, parity.E_FLOOR * A, "E")
    for lay, flag in ((amp.dense(n, cols), amp.ROWS_OPERAND0 | amp.rows_block(48)),       # 48 does not divide 256
                      (amp.dense(n, cols), amp.rows_block(B)),                              # no row-scaled operand
                      (amp.causal(1, rows, rows), amp.ROWS_OPERAND0 | amp.rows_block(8))):  # causal rows have no blocks
        d = amp.bgemm_desc(x, g, lay, None, None, amp.dense(0), R, ts, ti, None, None, scale_rows=flag)
        with pytest.raises(amp.AmpError) as ei:
            amp.amp_sens_bgemm_workspace_bytes([d], 2)
        assert ei.value.status == amp.ERR_INVALID_ARG
