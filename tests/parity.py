"""Comparison of one library pass (paper_2505_13060_amd.pipeline.SensPass) with the CPU
oracle on the same bytes.  Used by the GPU tests and the smoke check.

Bar: amax, scale and reciprocal scale bit-exact; FP8 codes bit-exact (test_gpu_fake_quant);
the fp32 sums within 1e-4 relative of the oracle's fp64 sums.  For E a floor of 1e-9 * A is
added: E is only meaningful relative to A * alpha_f (alpha >= 1/768), and an operand whose
elements all sit on the FP8 grid has a true E of order 1e-14 * A that fp32 cannot resolve.
When the oracle's sum is exactly zero the library's must be exactly zero.
"""
import numpy as np

import oracle
from paper_2505_13060_amd.workloads import to_bits

RTOL = 1e-4
E_FLOOR = 1e-9


def bits32(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def assert_sum_close(got, want, floor, what):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert np.all(np.isfinite(got)), what
    zero = want == 0
    assert np.all(got[zero] == 0), (what, got[zero])
    tol = RTOL * np.abs(want) + floor
    bad = np.abs(got - want) > tol
    assert not bad.any(), (what, got[bad][:4], want[bad][:4])


def oracle_scales(x_bits, fmts, causal=None, pow2=False):
    """(amax, scale, inv, flags) per format; pow2: the power-of-two scale rule instead of amax / FMAX."""
    out = []
    for f in fmts:
        am, sc, iv, fl = oracle.absmax_scale(x_bits, f, causal=causal)
        if pow2:
            sc, iv = oracle.scale_pow2(int(np.asarray(bits32(am)).reshape(-1)[0] >> 16), f)
        out.append((am, sc, iv, fl))
    return out


def check_scales(res, t, x_bits, fmts, causal, what):
    """Returns [(scale, inv)] per format after checking the library's values bit for bit."""
    ref = oracle_scales(x_bits, fmts, causal, pow2=res.get("pow2", False))
    assert bits32(res["amax"][t]) == bits32(ref[0][0]), (what, res["amax"][t], ref[0][0])
    assert res["flags"][t] == ref[0][3], what
    out = []
    for fi, (am, sc, iv, fl) in enumerate(ref):
        assert bits32(res["scale"][t, fi]) == bits32(sc), (what, fi, res["scale"][t, fi], sc)
        assert bits32(res["inv"][t, fi]) == bits32(iv), (what, fi, res["inv"][t, fi], iv)
        out.append((sc, iv))
    return out


def check_linear(op, k, res, fmts, samples=None):
    x, dx, w, dw = to_bits(op.x), to_bits(op.dx), to_bits(op.w), to_bits(op.dw)
    sx = check_scales(res, 2 * k, x.reshape(-1), fmts, None, op.name + ".x")
    sw = check_scales(res, 2 * k + 1, w.reshape(-1), fmts, None, op.name + ".w")
    got = res["linear"][k]                                   # [R, nf, 4]
    for fi, f in enumerate(fmts):
        want = oracle.sens_linear(x.reshape(-1), dx.reshape(-1), w.reshape(-1), dw.reshape(-1), op.C,
                                  op.K, op.R, op.row_offsets, sx[fi][0], sx[fi][1], sw[fi][0],
                                  sw[fi][1], f)
        rows = range(op.R) if samples is None else samples
        for r in rows:
            tag = "%s r=%d fmt=%d" % (op.name, r, f)
            assert_sum_close(got[r, fi, 1], want[r, 1], 0.0, tag + " A_X")
            assert_sum_close(got[r, fi, 3], want[r, 3], 0.0, tag + " A_W")
            assert_sum_close(got[r, fi, 0], want[r, 0], E_FLOOR * want[r, 1], tag + " E_X")
            assert_sum_close(got[r, fi, 2], want[r, 2], E_FLOOR * want[r, 3], tag + " E_W")


def _causal(lay):
    return None if lay[0] == "dense" else (lay[1], lay[2], lay[3])


def check_bgemm(op, k, n_linear, res, fmts):
    x0, dx0, x1, dx1 = to_bits(op.x0), to_bits(op.dx0), to_bits(op.x1), to_bits(op.dx1)
    t0 = 2 * n_linear + 2 * k

    def all_samples(lay):
        c = _causal(lay)
        return None if c is None else (c[0] * op.R, c[1], c[2])

    s0 = check_scales(res, t0, x0.reshape(-1), fmts, all_samples(op.lay0), op.name + ".x0")
    s1 = check_scales(res, t0 + 1, x1.reshape(-1), fmts, all_samples(op.lay1), op.name + ".x1")
    got = res["bgemm"][k]
    for fi, f in enumerate(fmts):
        want = oracle.sens_bgemm(x0.reshape(-1), dx0.reshape(-1), op.lay0, x1.reshape(-1),
                                 dx1.reshape(-1), op.lay1, op.R, s0[fi][0], s0[fi][1], s1[fi][0],
                                 s1[fi][1], f)
        for r in range(op.R):
            tag = "%s r=%d fmt=%d" % (op.name, r, f)
            assert_sum_close(got[r, fi, 1], want[r, 1], 0.0, tag + " A_0")
            assert_sum_close(got[r, fi, 3], want[r, 3], 0.0, tag + " A_1")
            assert_sum_close(got[r, fi, 0], want[r, 0], E_FLOOR * want[r, 1], tag + " E_0")
            assert_sum_close(got[r, fi, 2], want[r, 2], E_FLOOR * want[r, 3], tag + " E_1")


def check_workload(workload, res):
    for k, op in enumerate(workload.linears):
        check_linear(op, k, res, workload.fmts)
    for k, op in enumerate(workload.bgemms):
        check_bgemm(op, k, len(workload.linears), res, workload.fmts)


# ---- one scale per row (RowSensPass) ---------------------------------------------------------------

def _operand_scales(res, key, x_bits, n_rows, row_len, fmts, causal_rows, what):
    """Checks the library's scales of one operand bit for bit against the oracle and returns, per
    format, (scale[n_rows], inv[n_rows]); a per-tensor operand is broadcast to its rows."""
    w = res["where"][key]
    out = []
    if w[0] == "tensor":
        causal = None if causal_rows is None else (n_rows // causal_rows, causal_rows, row_len)
        for sc, iv in check_scales(res, w[1], x_bits, fmts, causal, what):
            out.append((np.full(n_rows, sc, dtype=np.float32), np.full(n_rows, iv, dtype=np.float32)))
        return out
    _, base, rows, ti = w
    assert rows == n_rows, (what, rows, n_rows)
    # scales computed by the sensitivity pass itself (single read) come without amax and flag words
    computed = key in res.get("computed", ())
    flags = 0
    for fi, f in enumerate(fmts):
        am, sc, iv, fl = oracle.absmax_scale_rows(x_bits, n_rows, row_len, f, causal_rows=causal_rows)
        flags |= fl
        if not computed:
            assert np.array_equal(bits32(res["row_amax"][base:base + n_rows]), bits32(am)), what
        assert np.array_equal(bits32(res["row_scale"][base:base + n_rows, fi]), bits32(sc)), (what, fi)
        assert np.array_equal(bits32(res["row_inv"][base:base + n_rows, fi]), bits32(iv)), (what, fi)
        out.append((sc, iv))
    if not computed:
        assert res["row_flags"][ti] == flags, what
    return out


def check_workload_rows(workload, res):
    fmts = workload.fmts
    for k, op in enumerate(workload.linears):
        x, dx, w, dw = (to_bits(t).reshape(-1) for t in (op.x, op.dx, op.w, op.dw))
        rows = int(op.row_offsets[-1])
        sx = _operand_scales(res, ("lin", k, 0), x, rows, op.C, fmts, None, op.name + ".x")
        sw = _operand_scales(res, ("lin", k, 1), w, op.K, op.C, fmts, None, op.name + ".w")
        got = res["linear"][k]
        for fi, f in enumerate(fmts):
            for r in range(op.R):
                r0, r1 = int(op.row_offsets[r]), int(op.row_offsets[r + 1])
                Ex, Ax = oracle.sens_operand_rows(x[r0 * op.C:r1 * op.C], dx[r0 * op.C:r1 * op.C], r1 - r0, op.C,
                                                  sx[fi][0][r0:r1], sx[fi][1][r0:r1], f)
                n = op.K * op.C
                Ew, Aw = oracle.sens_operand_rows(w, dw[r * n:(r + 1) * n], op.K, op.C, sw[fi][0], sw[fi][1], f)
                tag = "%s r=%d fmt=%d" % (op.name, r, f)
                assert_sum_close(got[r, fi, 1], Ax, 0.0, tag + " A_X")
                assert_sum_close(got[r, fi, 3], Aw, 0.0, tag + " A_W")
                assert_sum_close(got[r, fi, 0], Ex, E_FLOOR * Ax, tag + " E_X")
                assert_sum_close(got[r, fi, 2], Ew, E_FLOOR * Aw, tag + " E_W")
    for k, op in enumerate(workload.bgemms):
        got = res["bgemm"][k]
        sides = []
        for side, (xt, dxt, lay) in enumerate(((op.x0, op.dx0, op.lay0), (op.x1, op.dx1, op.lay1))):
            xb, db = to_bits(xt).reshape(-1), to_bits(dxt).reshape(-1)
            row_len = xt.shape[-1]
            causal_rows = lay[2] if lay[0] == "causal" else None
            n_rows = xb.size // row_len
            sc = _operand_scales(res, ("bg", k, side), xb, n_rows, row_len, fmts, causal_rows,
                                 "%s.x%d" % (op.name, side))
            sides.append((xb, db, row_len, causal_rows, n_rows // op.R, sc))
        for fi, f in enumerate(fmts):
            for r in range(op.R):
                vals = []
                for xb, db, row_len, causal_rows, per, sc in sides:
                    a, b = r * per, (r + 1) * per
                    vals.append(oracle.sens_operand_rows(xb[a * row_len:b * row_len], db[a * row_len:b * row_len],
                                                         per, row_len, sc[fi][0][a:b], sc[fi][1][a:b], f,
                                                         causal_rows=causal_rows))
                tag = "%s r=%d fmt=%d" % (op.name, r, f)
                assert_sum_close(got[r, fi, 1], vals[0][1], 0.0, tag + " A_0")
                assert_sum_close(got[r, fi, 3], vals[1][1], 0.0, tag + " A_1")
                assert_sum_close(got[r, fi, 0], vals[0][0], E_FLOOR * vals[0][1], tag + " E_0")
                assert_sum_close(got[r, fi, 2], vals[1][0], E_FLOOR * vals[1][1], tag + " E_1")


def _block_scales(res, key, x_bits, n_rows, row_len, block, fmts, what):
    """The library's scales of a dense operand cut into 1 x block tiles, bit for bit against the oracle's
    block routine; returns per format (scale, inv) as [n_rows, row_len // block] arrays."""
    _, base, rows, ti = res["where"][key]
    per = row_len // block
    assert rows == n_rows * per, (what, rows, n_rows, per)
    computed = key in res.get("computed", ())
    out, flags = [], 0
    for fi, f in enumerate(fmts):
        am, sc, iv, fl = oracle.absmax_scale_blocks(x_bits, n_rows, row_len, block, f)
        flags |= fl
        if not computed:
            assert np.array_equal(bits32(res["row_amax"][base:base + rows]), bits32(am.reshape(-1))), what
        assert np.array_equal(bits32(res["row_scale"][base:base + rows, fi]), bits32(sc.reshape(-1))), (what, fi)
        assert np.array_equal(bits32(res["row_inv"][base:base + rows, fi]), bits32(iv.reshape(-1))), (what, fi)
        out.append((sc, iv))
    if not computed:
        assert res["row_flags"][ti] == flags, what
    return out


def check_workload_blocks(workload, res, block):
    """Every operand with one scale per 1 x block tile of its dense rows (causal rows: one scale each):
    tables bit for bit, sums against the oracle's block routine."""
    fmts = workload.fmts
    for k, op in enumerate(workload.linears):
        x, dx, w, dw = (to_bits(t).reshape(-1) for t in (op.x, op.dx, op.w, op.dw))
        rows = int(op.row_offsets[-1])
        sx = _block_scales(res, ("lin", k, 0), x, rows, op.C, block, fmts, op.name + ".x")
        sw = _block_scales(res, ("lin", k, 1), w, op.K, op.C, block, fmts, op.name + ".w")
        got = res["linear"][k]
        n = op.K * op.C
        for fi, f in enumerate(fmts):
            for r in range(op.R):
                r0, r1 = int(op.row_offsets[r]), int(op.row_offsets[r + 1])
                Ex, Ax = oracle.sens_operand_blocks(x[r0 * op.C:r1 * op.C], dx[r0 * op.C:r1 * op.C], r1 - r0, op.C, block,
                                                    sx[fi][0][r0:r1], sx[fi][1][r0:r1], f)
                Ew, Aw = oracle.sens_operand_blocks(w, dw[r * n:(r + 1) * n], op.K, op.C, block, sw[fi][0], sw[fi][1], f)
                tag = "%s r=%d fmt=%d" % (op.name, r, f)
                assert_sum_close(got[r, fi, 1], Ax, 0.0, tag + " A_X")
                assert_sum_close(got[r, fi, 3], Aw, 0.0, tag + " A_W")
                assert_sum_close(got[r, fi, 0], Ex, E_FLOOR * Ax, tag + " E_X")
                assert_sum_close(got[r, fi, 2], Ew, E_FLOOR * Aw, tag + " E_W")
    for k, op in enumerate(workload.bgemms):
        got = res["bgemm"][k]
        vals = {}
        for side, (xt, dxt, lay) in enumerate(((op.x0, op.dx0, op.lay0), (op.x1, op.dx1, op.lay1))):
            xb, db = to_bits(xt).reshape(-1), to_bits(dxt).reshape(-1)
            row_len = xt.shape[-1]
            n_rows = xb.size // row_len
            per = n_rows // op.R
            what = "%s.x%d" % (op.name, side)
            if lay[0] == "causal":
                sc = _operand_scales(res, ("bg", k, side), xb, n_rows, row_len, fmts, lay[2], what)
                for fi, f in enumerate(fmts):
                    for r in range(op.R):
                        a, b = r * per, (r + 1) * per
                        vals[(side, fi, r)] = oracle.sens_operand_rows(xb[a * row_len:b * row_len], db[a * row_len:b * row_len], per,
                                                                       row_len, sc[fi][0][a:b], sc[fi][1][a:b], f, causal_rows=lay[2])
            else:
                sc = _block_scales(res, ("bg", k, side), xb, n_rows, row_len, block, fmts, what)
                for fi, f in enumerate(fmts):
                    for r in range(op.R):
                        a, b = r * per, (r + 1) * per
                        vals[(side, fi, r)] = oracle.sens_operand_blocks(xb[a * row_len:b * row_len], db[a * row_len:b * row_len], per,
                                                                         row_len, block, sc[fi][0][a:b], sc[fi][1][a:b], f)
        for fi, f in enumerate(fmts):
            for r in range(op.R):
                tag = "%s r=%d fmt=%d" % (op.name, r, f)
                assert_sum_close(got[r, fi, 1], vals[(0, fi, r)][1], 0.0, tag + " A_0")
                assert_sum_close(got[r, fi, 3], vals[(1, fi, r)][1], 0.0, tag + " A_1")
                assert_sum_close(got[r, fi, 0], vals[(0, fi, r)][0], E_FLOOR * vals[(0, fi, r)][1], tag + " E_0")
                assert_sum_close(got[r, fi, 2], vals[(1, fi, r)][0], E_FLOOR * vals[(1, fi, r)][1], tag + " E_1")
