"""GPU parity tests for one scale per row (per-token activations, per-channel weights, rows of
BGEMM operands): row amax and scales bit-exact, sums within 1e-4 of the oracle's per-row
routines (tests/parity.py).  Every test prints what it is about to run before touching the GPU."""
import ctypes as C
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2505_13060_amd as amp
from paper_2505_13060_amd import workloads as wl
from paper_2505_13060_amd.pipeline import RowSensPass, SensPass
from helpers import f32_to_bf16_bits
import parity

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def say(msg):
    print("[gpu-test] " + msg, flush=True)
    sys.stdout.flush()


def bf(bits, *shape):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).view(*shape)


def to_device(workload):
    for op in workload.linears:
        op.x, op.dx, op.w, op.dw = (t.to(DEV) for t in (op.x, op.dx, op.w, op.dw))
    for op in workload.bgemms:
        op.x0, op.dx0, op.x1, op.dx1 = (t.to(DEV) for t in (op.x0, op.dx0, op.x1, op.dx1))
    return workload


def run_rows(workload, **modes):
    say("rows %s: %s, %d linears, %d bgemms, %.1f M pairs" %
        (modes, workload.name, len(workload.linears), len(workload.bgemms), workload.pairs() / 1e6))
    to_device(workload)
    p = RowSensPass(workload, DEV, **modes)
    p.run()
    res = p.results()
    parity.check_workload_rows(workload, res)
    return p, res


def _mk(rng, n, sigma):
    return f32_to_bf16_bits((rng.standard_normal(n) * sigma).astype(np.float32))


@pytest.mark.parametrize("rows,row_len,off", [(700, 128, 0), (37, 11008, 0), (333, 100, 0), (300, 128, 6),
                                              (5000, 8, 0), (3, 28672, 0), (1, 40, 0), (129, 4096, 0), (64, 24, 0)])
def test_row_absmax_bit_exact_dense(rows, row_len, off):
    rng = np.random.default_rng(rows * 7 + row_len)
    x = f32_to_bf16_bits((rng.standard_normal((rows, row_len)) * np.exp(rng.normal(0, 2, (rows, 1)))).astype(np.float32))
    x[rows // 2] = 0                                         # an all-zero row: scale 1
    flat = x.reshape(-1)
    buf = torch.zeros(flat.size + 8, dtype=torch.int16, device=DEV)
    buf[off // 2: off // 2 + flat.size] = torch.from_numpy(flat.view(np.int16)).to(DEV)
    view = buf[off // 2:]
    fmts = [amp.E4M3, amp.E5M2]
    t = [amp.tensor(view, amp.dense(rows * row_len, row_len))]
    ws_bytes, n_rows = amp.amp_absmax_rows_workspace_bytes(t)
    assert n_rows == rows
    say("row absmax [%d, %d] offset %d" % (rows, row_len, off))
    d_amax = torch.zeros(rows, device=DEV)
    d_scale = torch.zeros(rows, 2, device=DEV)
    d_inv = torch.zeros(rows, 2, device=DEV)
    d_flags = torch.full((1,), 7, dtype=torch.int32, device=DEV)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=DEV)
    amp.amp_absmax_scale_rows(t, fmts, d_amax, d_scale, d_inv, d_flags, ws)
    torch.cuda.synchronize()
    assert int(d_flags[0]) == 0
    for fi, f in enumerate(fmts):
        am, sc, iv, fl = oracle.absmax_scale_rows(flat, rows, row_len, f)
        assert np.array_equal(parity.bits32(d_amax.cpu().numpy()), parity.bits32(am))
        assert np.array_equal(parity.bits32(d_scale[:, fi].cpu().numpy()), parity.bits32(sc))
        assert np.array_equal(parity.bits32(d_inv[:, fi].cpu().numpy()), parity.bits32(iv))


def test_row_absmax_causal_rows_many_tensors_and_flags():
    rng = np.random.default_rng(5)
    tensors, host = [], []
    for (b, r, c, samples) in [(2, 37, 48, 2), (1, 48, 24, 1), (3, 64, 64, 2), (1, 520, 512, 1), (2, 16, 72, 3)]:
        x = _mk(rng, samples * b * r * c, 0.5)
        i = np.arange(r)[:, None]
        j = np.arange(c)[None, :]
        outside = np.broadcast_to(j > i + (c - r), (samples * b, r, c)).reshape(-1)
        x[outside] = 0x7FC0                                  # NaN outside the operand: no effect
        tensors.append((x, b, r, c, samples))
    # a dense tensor with one Inf (flag), and an empty one
    xin = _mk(rng, 50 * 64, 1.0)
    xin[64 * 7 + 3] = 0x7F80
    dev = [torch.from_numpy(x.view(np.int16)).to(DEV) for (x, *_r) in tensors] + [torch.from_numpy(xin.view(np.int16)).to(DEV)]
    descs = [amp.tensor(d, amp.causal(b, r, c), s) for d, (x, b, r, c, s) in zip(dev, tensors)]
    descs.append(amp.tensor(dev[-1], amp.dense(50 * 64, 64)))
    descs.append(amp.tensor(None, amp.dense(0, 64)))
    ws_bytes, n_rows = amp.amp_absmax_rows_workspace_bytes(descs)
    want_rows = sum(s * b * r for (x, b, r, c, s) in tensors) + 50
    assert n_rows == want_rows
    say("row absmax, %d tensors, %d rows" % (len(descs), n_rows))
    fmts = [amp.E5M2]
    d_amax = torch.zeros(n_rows, device=DEV)
    d_scale = torch.zeros(n_rows, 1, device=DEV)
    d_inv = torch.zeros(n_rows, 1, device=DEV)
    d_flags = torch.full((len(descs),), 9, dtype=torch.int32, device=DEV)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=DEV)
    amp.amp_absmax_scale_rows(descs, fmts, d_amax, d_scale, d_inv, d_flags, ws)
    torch.cuda.synchronize()
    flags = d_flags.cpu().numpy()
    assert list(flags) == [0, 0, 0, 0, 0, 1, 0]
    base = 0
    am_g, sc_g, iv_g = d_amax.cpu().numpy(), d_scale.cpu().numpy()[:, 0], d_inv.cpu().numpy()[:, 0]
    for (x, b, r, c, s) in tensors:
        n = s * b * r
        am, sc, iv, fl = oracle.absmax_scale_rows(x, n, c, amp.E5M2, causal_rows=r)
        assert fl == 0
        assert np.array_equal(parity.bits32(am_g[base:base + n]), parity.bits32(am))
        assert np.array_equal(parity.bits32(sc_g[base:base + n]), parity.bits32(sc))
        assert np.array_equal(parity.bits32(iv_g[base:base + n]), parity.bits32(iv))
        base += n
    am, sc, iv, fl = oracle.absmax_scale_rows(xin, 50, 64, amp.E5M2)
    assert fl == 1
    ok = np.arange(50) != 7
    assert np.array_equal(parity.bits32(am_g[base:base + 50])[ok], parity.bits32(am)[ok])
    assert np.isinf(am_g[base + 7])


def test_rows_config0_full():
    run_rows(wl.config0("cpu"))


def test_rows_config1_reduced_block_all_rows():
    run_rows(wl.config1("cpu", R=3, S=200, hidden=520, ffn=1384, H=4, D=64))


@pytest.mark.parametrize("modes", [dict(x_rows=True, w_rows=False, bgemm_rows=False),
                                   dict(x_rows=False, w_rows=True, bgemm_rows=False),
                                   dict(x_rows=False, w_rows=False, bgemm_rows=True)])
def test_rows_mixed_with_per_tensor_operands(modes):
    run_rows(wl.config1("cpu", R=2, S=136, hidden=256, ffn=520, H=2, D=64), **modes)


def test_rows_one_call_for_linears_and_bgemms():
    """Row scales through amp_sens_block: four classes of units in one call."""
    w = wl.config1("cpu", R=3, S=200, hidden=520, ffn=1384, H=4, D=64)
    p_one, res_one = run_rows(w, one_call=True)
    p_two, res_two = run_rows(w)
    for key in ("linear", "bgemm"):
        for a, b in zip(res_one[key], res_two[key]):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


@pytest.mark.parametrize("single_read,block", [(False, 0), (True, 0), (True, 128)])
def test_rows_config2_block_at_full_size_every_unit(single_read, block):
    """One whole block of the benchmark's workload with one scale per row on every operand (per token,
    per output channel, per row of the BGEMM operands), in the launch configurations
    `bench.py --scales rows` (two passes) and `bench.py --scales rows-single-read` (the pass that
    derives the row scales itself) time: every row's scales bit for bit and every (op, operand,
    sample, format) sum against the oracle, fanned over host threads.  block = 128: one scale per
    1 x 128 tile of every dense row (`--scale-block 128`), causal rows one scale each."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    which = (3 if single_read else 2) if block == 0 else 0
    say("rows%s%s, config2 block %d (one of the blocks bench.py times) at full size: generating on the GPU" %
        (", single read" if single_read else "", ", 1 x %d tiles" % block if block else "", which))
    w = wl.config2_block(DEV, which)
    torch.cuda.synchronize()
    p = RowSensPass(w, DEV, one_call=True, single_read=single_read, block=block)
    p.run()

    def scales_of(key, bits, n_rows, row_len, causal_rows, what):
        if block and causal_rows is None:
            return parity._block_scales(res, key, bits, n_rows, row_len, block, fmts, what)
        return parity._operand_scales(res, key, bits, n_rows, row_len, fmts, causal_rows, what)

    res = p.results()
    fmts = w.fmts
    units = []                  # (tag, got [nf, 2], x, dx, n_rows, row_len, causal_rows, scales of those rows)
    for k, op in enumerate(w.linears):
        say("  %s: copying to the host, scales of every row" % op.name)
        x, dx, wt, dw = (wl.to_bits(t).reshape(-1) for t in (op.x, op.dx, op.w, op.dw))
        rows = int(op.row_offsets[-1])
        sx = scales_of(("lin", k, 0), x, rows, op.C, None, op.name + ".x")
        sw = scales_of(("lin", k, 1), wt, op.K, op.C, None, op.name + ".w")
        n = op.K * op.C
        for r in range(op.R):
            r0, r1 = int(op.row_offsets[r]), int(op.row_offsets[r + 1])
            units.append(("%s.X r=%d" % (op.name, r), res["linear"][k][r][:, 0:2], x[r0 * op.C:r1 * op.C],
                          dx[r0 * op.C:r1 * op.C], r1 - r0, op.C, None, [(a[r0:r1], b[r0:r1]) for a, b in sx]))
            units.append(("%s.W r=%d" % (op.name, r), res["linear"][k][r][:, 2:4], wt, dw[r * n:(r + 1) * n],
                          op.K, op.C, None, sw))
    for k, op in enumerate(w.bgemms):
        for side, (xt, dxt, lay) in enumerate(((op.x0, op.dx0, op.lay0), (op.x1, op.dx1, op.lay1))):
            say("  %s operand %d: copying to the host, scales of every row" % (op.name, side))
            xb, db = wl.to_bits(xt).reshape(-1), wl.to_bits(dxt).reshape(-1)
            row_len = xt.shape[-1]
            causal_rows = lay[2] if lay[0] == "causal" else None
            n_rows = xb.size // row_len
            sc = scales_of(("bg", k, side), xb, n_rows, row_len, causal_rows, "%s.x%d" % (op.name, side))
            per = n_rows // op.R
            for r in range(op.R):
                a, b = r * per, (r + 1) * per
                units.append(("%s.x%d r=%d" % (op.name, side, r), res["bgemm"][k][r][:, 2 * side:2 * side + 2],
                              xb[a * row_len:b * row_len], db[a * row_len:b * row_len], per, row_len, causal_rows,
                              [(s_[a:b], i_[a:b]) for s_, i_ in sc]))

    def one(u):
        tag, got, xb, gb, n_rows, row_len, causal_rows, sc = u
        for fi, f in enumerate(fmts):
            if block and causal_rows is None:
                E, A = oracle.sens_operand_blocks(xb, gb, n_rows, row_len, block, sc[fi][0], sc[fi][1], f)
            else:
                E, A = oracle.sens_operand_rows(xb, gb, n_rows, row_len, sc[fi][0], sc[fi][1], f, causal_rows=causal_rows)
            parity.assert_sum_close(got[fi, 1], A, 0.0, tag + " A fmt=%d" % f)
            parity.assert_sum_close(got[fi, 0], E, parity.E_FLOOR * A, tag + " E fmt=%d" % f)
        return tag

    threads = max(1, min(16, os.cpu_count() or 1))
    say("  %d units on %d host threads" % (len(units), threads))
    with ThreadPoolExecutor(threads) as ex:
        for i, tag in enumerate(ex.map(one, units)):
            if i % 32 == 31:
                say("  ... %d units match, last %s" % (i + 1, tag))
    assert len(units) == 16 * 2 * (len(w.linears) + len(w.bgemms))


def test_rows_config3_reduced_single_format():
    run_rows(wl.config3("cpu", R=2, S=264, hidden=512, ffn=1800, Hq=8, Hkv=2, D=64))


def test_rows_config4_reduced_ragged_many_small():
    run_rows(wl.config4("cpu", R=5, experts=6, C=512, K=176, tok_lo=1, tok_hi=40, n_bgemm=4, S=72, H=2, D=32))


def test_rows_weight_kernel_on_and_off():
    for (R, tokens, Cd, K) in [(11, 40, 520, 190), (3, 16, 1024, 100), (2, 64, 4096, 24), (9, 24, 40, 2500)]:
        w = wl.Workload("wk_rows", [amp.E4M3, amp.E5M2],
                        [wl._linear("lin", 555 + R, R, tokens, Cd, K, "cpu", outliers=2)])
        outs = []
        for on in (0, 1):
            say("weight kernel %s with row scales: R=%d W=%dx%d" % ("on" if on else "off", R, K, Cd))
            p, res = run_rows(w, plan=True, flags=0 if on else amp.PLAN_STREAM_WEIGHTS)
            outs.append(res["linear"][0].copy())
        assert np.allclose(outs[0], outs[1], rtol=2e-6, atol=0)


def test_rows_odd_row_lengths_misalignment_and_causal_shapes():
    rng = np.random.default_rng(123)
    lin, bg = [], []
    # C not a multiple of 8 (element path), empty and one-token samples
    off = np.array([0, 0, 1, 1, 40], dtype=np.int64)
    Cd, K, R = 52, 9, 4
    lin.append(wl.LinearOp("odd_C", bf(_mk(rng, 40 * Cd, 1.0), 40, Cd), bf(_mk(rng, 40 * Cd, 1e-3), 40, Cd),
                           bf(_mk(rng, K * Cd, 0.02), K, Cd), bf(_mk(rng, R * K * Cd, 1e-3), R, K, Cd), R, Cd, K, off))
    # short rows: several rows per vector step
    Cd, K, R = 8, 300, 2
    lin.append(wl.LinearOp("C8", bf(_mk(rng, 2 * 50 * Cd, 1.0), 100, Cd), bf(_mk(rng, 100 * Cd, 1e-3), 100, Cd),
                           bf(_mk(rng, K * Cd, 0.02), K, Cd), bf(_mk(rng, R * K * Cd, 1e-3), R, K, Cd), R, Cd, K,
                           np.array([0, 50, 100], dtype=np.int64)))
    for (H, S, S2, D) in [(2, 37, 48, 24), (1, 48, 24, 8), (3, 33, 33, 40), (2, 16, 16, 16), (1, 136, 136, 64), (2, 40, 64, 12)]:
        R = 2
        p, dp = _mk(rng, R * H * S * S2, 0.3), _mk(rng, R * H * S * S2, 1e-3)
        i = np.arange(S)[:, None]
        j = np.arange(S2)[None, :]
        outside = np.broadcast_to(j > i + (S2 - S), (R * H, S, S2)).reshape(-1)
        p[outside] = 0x7FC0
        dp[outside] = 0xFFC0
        v, dv = _mk(rng, R * H * S2 * D, 1.0), _mk(rng, R * H * S2 * D, 1e-3)
        bg.append(wl.BgemmOp("odd_causal_%dx%d" % (S, S2), bf(p, R, H, S, S2), bf(dp, R, H, S, S2), ("causal", H, S, S2),
                             bf(v, R, H, S2, D), bf(dv, R, H, S2, D), ("dense", H * S2 * D), R))
    run_rows(wl.Workload("edge_rows", [amp.E4M3, amp.E5M2], lin, bg))


def test_rows_with_equal_rows_reproduce_the_per_tensor_pass():
    """If every row of an operand has the same amax, the per-row pass must give the per-tensor sums."""
    w = wl.config1("cpu", R=2, S=64, hidden=128, ffn=256, H=2, D=32)
    peak = f32_to_bf16_bits(np.array([4096.0], dtype=np.float32)).view(np.int16)[0]
    for op in w.linears:
        op.x.view(torch.int16)[:, 0] = int(peak)
        op.w.view(torch.int16)[:, 0] = int(peak)
    to_device(w)
    say("rows vs per-tensor on equal-amax rows")
    a = RowSensPass(w, DEV, bgemm_rows=False)
    a.run()
    ra = a.results()
    b = SensPass(w, DEV)
    b.run()
    rb = b.results()
    for k in range(len(w.linears)):
        assert np.allclose(ra["linear"][k], rb["linear"][k], rtol=3e-6, atol=0), w.linears[k].name
    for k in range(len(w.bgemms)):
        assert np.array_equal(ra["bgemm"][k], rb["bgemm"][k])


def test_power_of_two_scales_per_tensor_and_per_row_bit_exact():
    """AMP_SCALE_POW2: the smallest power of two that fits amax into the format, against the oracle, for
    magnitudes over the whole bf16 range including amax = FMAX * 2^k exactly and its neighbours; then the
    sums at those scales against the oracle."""
    rng = np.random.default_rng(77)
    rows, row_len = 600, 64
    x = f32_to_bf16_bits((rng.standard_normal((rows, row_len)) * np.exp(rng.uniform(-80, 80, (rows, 1)))).astype(np.float32))
    exact = f32_to_bf16_bits(np.array([448.0 * 2.0 ** k for k in range(-60, 60)], dtype=np.float32))
    for i, h in enumerate(exact):                              # rows whose amax is FMAX * 2^k, one step above, one below
        x[3 * i] = 0
        x[3 * i, 5] = h
        x[3 * i + 1] = 0
        x[3 * i + 1, 7] = h + 1
        x[3 * i + 2] = 0
        x[3 * i + 2, 9] = h - 1
    x[590] = 0                                                 # amax = 0
    x[591] = 1                                                 # the smallest subnormal: no fp32 reciprocal
    flat = x.reshape(-1)
    d = torch.from_numpy(flat.view(np.int16)).to(DEV)
    fmts = [amp.E4M3 | amp.SCALE_POW2, amp.E5M2 | amp.SCALE_POW2]
    t = [amp.tensor(d, amp.dense(rows * row_len, row_len))]
    ws_bytes, n_rows = amp.amp_absmax_rows_workspace_bytes(t)
    say("power-of-two scales, %d rows" % n_rows)
    d_amax = torch.zeros(rows, device=DEV)
    d_scale = torch.zeros(rows, 2, device=DEV)
    d_inv = torch.zeros(rows, 2, device=DEV)
    d_flags = torch.zeros(1, dtype=torch.int32, device=DEV)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=DEV)
    amp.amp_absmax_scale_rows(t, fmts, d_amax, d_scale, d_inv, d_flags, ws)
    torch.cuda.synchronize()
    am = d_amax.cpu().numpy()
    am_bits = (parity.bits32(am) >> 16).astype(np.uint16)
    assert np.array_equal(am_bits, (flat.reshape(rows, row_len) & 0x7FFF).max(axis=1))
    for fi, f in enumerate([amp.E4M3, amp.E5M2]):
        want = [oracle.scale_pow2(h, f) for h in am_bits]
        assert np.array_equal(parity.bits32(d_scale[:, fi].cpu().numpy()), parity.bits32(np.array([w[0] for w in want])))
        assert np.array_equal(parity.bits32(d_inv[:, fi].cpu().numpy()), parity.bits32(np.array([w[1] for w in want])))
    # per tensor, several tensors in one call
    tens = [amp.tensor(d[i * row_len:], amp.dense(row_len * 10)) for i in (0, 3, 30, 300, 590)]
    ws2 = torch.empty(max(amp.amp_absmax_workspace_bytes(tens), 256), dtype=torch.uint8, device=DEV)
    a2 = torch.zeros(5, device=DEV)
    s2 = torch.zeros(5, 2, device=DEV)
    i2 = torch.zeros(5, 2, device=DEV)
    f2 = torch.zeros(5, dtype=torch.int32, device=DEV)
    amp.amp_absmax_scale(tens, fmts, a2, s2, i2, f2, ws2)
    torch.cuda.synchronize()
    for j, i in enumerate((0, 3, 30, 300, 590)):
        h = int((flat[i * row_len:(i + 10) * row_len] & 0x7FFF).max())
        for fi, f in enumerate([amp.E4M3, amp.E5M2]):
            sc, iv = oracle.scale_pow2(h, f)
            assert parity.bits32(s2[j, fi].cpu().numpy()) == parity.bits32(sc)
            assert parity.bits32(i2[j, fi].cpu().numpy()) == parity.bits32(iv)
    # the sums at power-of-two row scales (magnitudes that keep the fp32 sums finite)
    x2 = f32_to_bf16_bits((rng.standard_normal((rows, row_len)) * np.exp(rng.uniform(-8, 8, (rows, 1)))).astype(np.float32)).reshape(-1)
    g = f32_to_bf16_bits((rng.standard_normal(rows * row_len) * 1e-2).astype(np.float32))
    dx2 = torch.from_numpy(x2.view(np.int16)).to(DEV)
    dg = torch.from_numpy(g.view(np.int16)).to(DEV)
    t2 = [amp.tensor(dx2, amp.dense(rows * row_len, row_len))]
    amp.amp_absmax_scale_rows(t2, fmts, d_amax, d_scale, d_inv, d_flags, ws)
    desc = [amp.bgemm_desc(dx2, dg, amp.dense(rows * row_len, row_len), dx2, dg, amp.dense(rows * row_len, row_len), 1,
                           d_scale, d_inv, d_scale, d_inv, scale_rows=amp.ROWS_OPERAND0 | amp.ROWS_OPERAND1)]
    out = torch.zeros(1, 2, 4, device=DEV)
    ws3 = torch.empty(max(amp.amp_sens_bgemm_workspace_bytes(desc, 2), 256), dtype=torch.uint8, device=DEV)
    amp.amp_sens_bgemm(desc, [amp.E4M3, amp.E5M2], out, ws3)
    torch.cuda.synchronize()
    got = out.cpu().numpy()[0]
    for fi, f in enumerate([amp.E4M3, amp.E5M2]):
        sc = d_scale[:, fi].cpu().numpy()
        iv = d_inv[:, fi].cpu().numpy()
        assert np.all(np.log2(sc) == np.round(np.log2(sc)))
        E, A = oracle.sens_operand_rows(x2, g, rows, row_len, sc, iv, f)
        parity.assert_sum_close(got[fi, 1], A, 0.0, "A pow2 fmt=%d" % f)
        parity.assert_sum_close(got[fi, 0], E, parity.E_FLOOR * A, "E pow2 fmt=%d" % f)
        parity.assert_sum_close(got[fi, 3], A, 0.0, "A1 pow2 fmt=%d" % f)
        parity.assert_sum_close(got[fi, 2], E, parity.E_FLOOR * A, "E1 pow2 fmt=%d" % f)
