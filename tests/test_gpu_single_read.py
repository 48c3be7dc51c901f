"""The single-read form of the pass with one scale per row (AMP_ROWS_COMPUTE0 / 1): the sensitivity
pass finds each row's absmax itself, derives the scales and casts the row from registers.  The
scale tables it writes must equal the oracle's per-row scales bit for bit (both scale rules, every
special case of the scale arithmetic), the sums must match the oracle's row-scaled sums, for every row
geometry the kernel has: 4 to 256 threads per row, 4 to 12 vectors per thread, rows that span several
waves, ragged last tiles, causal rows whose lanes follow their length."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2505_13060_amd as amp
from paper_2505_13060_amd import workloads as wl
from paper_2505_13060_amd.pipeline import RowSensPass
from helpers import f32_to_bf16_bits
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


def run(workload, **modes):
    say("single read %s: %s, %d linears, %d bgemms, %.1f M pairs" %
        (modes, workload.name, len(workload.linears), len(workload.bgemms), workload.pairs() / 1e6))
    to_device(workload)
    p = RowSensPass(workload, DEV, single_read=True, **modes)
    p.r_scale.fill_(float("nan"))
    p.r_inv.fill_(float("nan"))
    p.run()
    res = p.results()
    parity.check_workload_rows(workload, res)
    return p, res


def test_single_read_reduced_blocks():
    run(wl.config1("cpu", R=3, S=136, hidden=256, ffn=520, H=2, D=64))
    run(wl.config3("cpu", R=2, S=264, hidden=512, ffn=1800, Hq=8, Hkv=2, D=64), one_call=True)
    run(wl.config4("cpu", R=5, experts=6, C=512, K=176, tok_lo=1, tok_hi=40, n_bgemm=4, S=72, H=2, D=32), plan=True)


@pytest.mark.parametrize("C", [8, 32, 64, 128, 136, 256, 1024, 4096, 8192, 11008, 16392, 24576])
def test_single_read_row_lengths(C):
    """Rows from one vector to the longest a workgroup can stage (12 vectors per thread); token counts
    that leave a ragged last tile; a sample without tokens."""
    R, K = 3, 8
    off = np.array([0, 37, 37, 37 + (5 if C > 8192 else 70)], dtype=np.int64)
    w = wl.Workload("rows_%d" % C, [amp.E4M3, amp.E5M2],
                    [wl._linear("lin", 9000 + C, R, 0, C, K, "cpu", outliers=max(1, C // 100), row_offsets=off)])
    run(w)


@pytest.mark.parametrize("row_len", [32, 64, 128, 256])
@pytest.mark.parametrize("rule", [0, amp.SCALE_POW2])
def test_single_read_short_rows_over_many_tiles(row_len, rule):
    """Short power-of-two rows take the tiles of 1024 consecutive vectors (one lane per vector, four rows per
    thread): row counts that fill several chunks, end in the middle of a tile, in the middle of a wave, and
    a sample of a single row; every row's scales bit for bit, sums against the oracle."""
    rng = np.random.default_rng(7 * row_len + rule)
    for rows in (1, 3 * (1 << 16) // row_len + 5, 20000):
        R = 2
        n = rows * row_len
        mags = np.exp(rng.uniform(-3, 3, (R * rows, 1)))
        x = f32_to_bf16_bits((rng.standard_normal((R * rows, row_len)) * mags).astype(np.float32)).reshape(-1)
        g = f32_to_bf16_bits((rng.standard_normal(R * n) * 1e-2).astype(np.float32))
        X = torch.from_numpy(x.view(np.int16)).to(DEV)
        G = torch.from_numpy(g.view(np.int16)).to(DEV)
        ts = torch.full((R * rows, 2), float("nan"), device=DEV)
        ti = torch.full((R * rows, 2), float("nan"), device=DEV)
        fmts_plain = [amp.E4M3, amp.E5M2]
        d = amp.bgemm_desc(X, G, amp.dense(n, row_len), None, None, amp.dense(0), R, ts, ti, None, None,
                           scale_rows=amp.ROWS_COMPUTE0)
        out = torch.zeros(R, 2, 4, device=DEV)
        ws = torch.empty(amp.amp_sens_bgemm_workspace_bytes([d], 2), dtype=torch.uint8, device=DEV)
        say("short rows of %d, %d rows per sample, rule %#x" % (row_len, rows, rule))
        amp.amp_sens_bgemm([d], [f | rule for f in fmts_plain], out, ws)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        for fi, f in enumerate(fmts_plain):
            am, sc, iv, _ = oracle.absmax_scale_rows(x, R * rows, row_len, f)
            if rule:
                both = [oracle.scale_pow2(int(b), f) for b in (parity.bits32(am) >> 16)]
                sc = np.array([b_[0] for b_ in both], dtype=np.float32)
                iv = np.array([b_[1] for b_ in both], dtype=np.float32)
            assert np.array_equal(parity.bits32(ts[:, fi].cpu().numpy()), parity.bits32(sc)), (fi, "scale")
            assert np.array_equal(parity.bits32(ti[:, fi].cpu().numpy()), parity.bits32(iv)), (fi, "inv")
            for r in range(R):
                E, A = oracle.sens_operand_rows(x[r * n:(r + 1) * n], g[r * n:(r + 1) * n], rows, row_len,
                                                sc[r * rows:(r + 1) * rows], iv[r * rows:(r + 1) * rows], f)
                parity.assert_sum_close(got[r, fi, 1], A, 0.0, "A fmt %d sample %d" % (f, r))
                parity.assert_sum_close(got[r, fi, 0], E, parity.E_FLOOR * A, "E fmt %d sample %d" % (f, r))


def test_single_read_rejects_rows_it_cannot_stage():
    n = 40
    d = amp.BgemmDesc()
    d.x0 = d.dx0 = d.x1 = d.dx1 = 4096
    d.scale0 = d.inv0 = d.scale1 = d.inv1 = 4096
    d.R = 1
    size = torch.zeros(1, device=DEV)                       # touches the GPU only to be a GPU test like its neighbours
    for cols, ok in ((24576, True), (24584, False), (100, False)):
        d.layout0, d.layout1 = amp.dense(n * cols, cols), amp.dense(0)
        d.scale_rows = amp.ROWS_COMPUTE0
        if ok:
            assert amp.amp_sens_bgemm_workspace_bytes([d], 2) > 0
        else:
            with pytest.raises(amp.AmpError) as ei:
                amp.amp_sens_bgemm_workspace_bytes([d], 2)
            assert ei.value.status == amp.ERR_INVALID_ARG
    d.layout0, d.scale_rows = amp.dense(n * 64, 64), amp.ROWS_COMPUTE0
    d.x0 = 4098                                             # not 16-byte aligned
    with pytest.raises(amp.AmpError):
        amp.amp_sens_bgemm_workspace_bytes([d], 2)
    lin = amp.LinearDesc()
    lin.x = lin.dx = lin.w = lin.dw = 4096
    lin.x_scale = lin.x_inv = lin.w_scale = lin.w_inv = 4096
    lin.C, lin.K, lin.tokens, lin.R = 64, 8, 4, 1
    lin.scale_rows = amp.ROWS_COMPUTE1                      # a weight's scales are not computed by the pass
    with pytest.raises(amp.AmpError):
        amp.amp_sens_linear_workspace_bytes([lin], 2)
    del size


@pytest.mark.parametrize("rule", [0, amp.SCALE_POW2])
@pytest.mark.parametrize("row_len,causal", [(64, False), (4096, False), (128, True)])
def test_single_read_scale_arithmetic_special_cases(rule, row_len, causal):
    """Rows whose absmax spans the whole bf16 range: zero rows, subnormal rows, rows whose reciprocal
    scale overflows fp32 (scale and reciprocal then both 1), amax = FMAX * 2^k and its neighbours, the
    largest finite value; with amax / FMAX scales and with power-of-two scales.  Tables bit for bit,
    sums against the oracle at those scales (gradients sized so that the fp32 sums stay finite)."""
    rng = np.random.default_rng(row_len + rule)
    rows = 512 if causal else 640
    mags = np.exp(rng.uniform(-85, 85, (rows, 1)))
    x = f32_to_bf16_bits((rng.standard_normal((rows, row_len)) * mags).astype(np.float32))
    special = [0x0000, 0x0001, 0x007F, 0x0080, 0x03DF, 0x03E0, 0x03E1, 0x075F, 0x0760, 0x0761, 0x7F7F, 0x7F00]
    special += [int(f32_to_bf16_bits(np.array([448.0 * 2.0 ** k], dtype=np.float32))[0]) + d for k in (-60, -7, 0, 9, 60)
                for d in (-1, 0, 1)]
    special += [int(f32_to_bf16_bits(np.array([57344.0 * 2.0 ** k], dtype=np.float32))[0]) + d for k in (-60, 0, 30)
                for d in (-1, 0, 1)]
    # gradients sized against the row's magnitude, so that every row's (xdot * x)^2 is of order 1e-6
    g = f32_to_bf16_bits((rng.standard_normal((rows, row_len)) * 1e-3 / mags).astype(np.float32))
    for i, h in enumerate(special):                          # a row whose only non-zero entry is the special value
        r = 20 + 7 * i
        valid = (r % row_len) + 1 if causal else row_len
        x[r, :valid] = 0
        x[r, (3 * i) % valid] = h ^ (0x8000 if i % 2 else 0)
        e = (h >> 7) & 0xFF
        g[r] = f32_to_bf16_bits(np.array([2.0 ** (127 - max(e, 1)) * 1e-3], dtype=np.float32))[0]
    fmts_plain = [amp.E4M3, amp.E5M2]
    fmts = [f | rule for f in fmts_plain]
    X = torch.from_numpy(x.reshape(-1).view(np.int16)).to(DEV)
    G = torch.from_numpy(g.reshape(-1).view(np.int16)).to(DEV)
    if causal:
        assert rows % row_len == 0
        lay = amp.causal(rows // row_len, row_len, row_len)
        causal_rows = row_len
    else:
        lay = amp.dense(rows * row_len, row_len)
        causal_rows = None
    ts = torch.full((rows, 2), float("nan"), device=DEV)
    ti = torch.full((rows, 2), float("nan"), device=DEV)
    d = amp.bgemm_desc(X, G, lay, None, None, amp.dense(0), 1, ts, ti, None, None, scale_rows=amp.ROWS_COMPUTE0)
    out = torch.zeros(1, 2, 4, device=DEV)
    ws = torch.empty(amp.amp_sens_bgemm_workspace_bytes([d], 2), dtype=torch.uint8, device=DEV)
    say("scale special cases: rows of %d, causal=%s, rule=%#x" % (row_len, causal, rule))
    amp.amp_sens_bgemm([d], fmts, out, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy()[0]
    xb, gb = x.reshape(-1), g.reshape(-1)
    for fi, f in enumerate(fmts_plain):
        if rule:
            i_idx = np.arange(row_len)[None, :] <= (np.arange(rows) % row_len)[:, None] if causal else np.ones((rows, row_len), bool)
            am_bits = np.where(i_idx, x & 0x7FFF, 0).max(axis=1)
            want = [oracle.scale_pow2(int(h), f) for h in am_bits]
            sc = np.array([w_[0] for w_ in want], dtype=np.float32)
            iv = np.array([w_[1] for w_ in want], dtype=np.float32)
        else:
            _, sc, iv, _ = oracle.absmax_scale_rows(xb, rows, row_len, f, causal_rows=causal_rows)
        assert np.array_equal(parity.bits32(ts[:, fi].cpu().numpy()), parity.bits32(sc)), (fi, "scale")
        assert np.array_equal(parity.bits32(ti[:, fi].cpu().numpy()), parity.bits32(iv)), (fi, "inv")
        E, A = oracle.sens_operand_rows(xb, gb, rows, row_len, sc, iv, f, causal_rows=causal_rows)
        parity.assert_sum_close(got[fi, 1], A, 0.0, "A fmt %d" % f)
        parity.assert_sum_close(got[fi, 0], E, parity.E_FLOOR * A, "E fmt %d" % f)
