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


def oracle_scales(x_bits, fmts, causal=None):
    out = []
    for f in fmts:
        out.append(oracle.absmax_scale(x_bits, f, causal=causal))
    return out


def check_scales(res, t, x_bits, fmts, causal, what):
    """Returns [(scale, inv)] per format after checking the library's values bit for bit."""
    ref = oracle_scales(x_bits, fmts, causal)
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
