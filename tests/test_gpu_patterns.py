"""Every bf16 pattern through every fused sensitivity kernel, one element at a time.

The fused kernels hold several copies of the FP8 cast (streaming, row-scaled, weight kernel), and
their codes can only be seen through sums.  Here every (op, sample) of a call has exactly one
element whose gradient is not zero, so its E is that one element's xdot^2 (x - xtilde)^2 and a
single wrong code anywhere fails: the sums of 65 536 such samples (all bf16 patterns) are compared
with the oracle's value for the same one-element operand.  Elements with a zero gradient add
exactly zero on both sides.

Layout trick that keeps this small: every op reads a window of one pattern buffer (the windows of
op k start 8 k elements in) and all ops share one gradient buffer, so 8 192 ops x 8 samples sweep
all patterns with a few hundred KB of operands.  Four value ranges (with matching scales and
gradient magnitudes) cover all finite bf16 values without leaving the fp32 range of the sums.
"""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2505_13060_amd as amp
from helpers import all_bf16_patterns, f32_to_bf16_bits
import parity

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
FMTS = [amp.E4M3, amp.E5M2]
R = 8
N_OPS = 8192
G_BASE = np.array([1.0, -2.0, 0.5, 3.0, -1.0, 1.5, 2.0, -0.75], dtype=np.float32)
ROW_MULT = np.array([1.0, 1.25, 0.75, 1.5, 0.625, 0.875, 1.125, 2.0], dtype=np.float32)

# value ranges: bf16 exponent fields [lo, hi] that stay, amax the scales are derived from (None:
# scale = inv = 1), power of two applied to the gradients
RANGES = {
    "unit_scale": dict(lo=87, hi=167, amax=None, gexp=0),
    "amax_3.1416": dict(lo=87, hi=167, amax=3.1416, gexp=0),
    "tiny": dict(lo=0, hi=86, amax=1.3 * 2.0 ** -90, gexp=100),
    "huge": dict(lo=168, hi=254, amax=1.7 * 2.0 ** 100, gexp=-100),
}


# value ranges for the scaled-conversion paths: a power-of-two scale s (reciprocal 1 / s) and only values
# up to FMAX * s in magnitude, which is what the flag on the sensitivity call promises
RANGES_POW2 = {
    "pow2_unit": dict(lo=87, hi=134, scale=1.0, gexp=0),
    "pow2_tiny": dict(lo=0, hi=86, scale=2.0 ** -48, gexp=100),
    # the top values round to 256 s = 2^128, which fp32 does not hold, while x - 2^128 is an ordinary number
    "pow2_huge": dict(lo=168, hi=254, scale=2.0 ** 120, gexp=-100),
}


def say(msg):
    print("[gpu-test] " + msg, flush=True)
    sys.stdout.flush()


def dev_bits(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV)


def scales_of(rng_name):
    """[(scale, inv)] per format as float32."""
    if rng_name in RANGES_POW2:
        s_ = np.float32(RANGES_POW2[rng_name]["scale"])
        return [(s_, np.float32(1.0) / s_) for _ in FMTS]
    amax = RANGES[rng_name]["amax"]
    out = []
    for f in FMTS:
        if amax is None:
            out.append((np.float32(1.0), np.float32(1.0)))
        else:
            fm, am = np.float32(oracle.fp8_max(f)), np.float32(amax)
            out.append((np.float32(am / fm), np.float32(fm / am)))
    return out


def patterns_of(rng_name):
    h = all_bf16_patterns().copy()
    e = (h >> 7) & 0xFF
    rg = RANGES_POW2[rng_name] if rng_name in RANGES_POW2 else RANGES[rng_name]
    keep = (e >= rg["lo"]) & (e <= rg["hi"])
    h[~keep] = 0
    return h


# ---- the kernel paths ---------------------------------------------------------------------------
# Each returns (n0 = elements per sample block, hot element h_r of sample r inside its block,
# row of that element inside the sample or None, rows per sample, layout, misalignment of x in
# elements, kind of op)

def hot_dense(r):
    return 8 * ((531 * r + 77) % 4096) + r


def hot_causal(r):                     # entry (i, j) of a [128, 128] lower triangle, j <= i
    i, j = 40 + 11 * r, 8 * ((3 * r + 1) % 5) + r
    assert j <= i
    return i * 128 + j, i


PATHS = {
    # streaming kernel, one scale per tensor
    "dense": dict(n0=32768, hot=hot_dense, layout=lambda: amp.dense(32768)),
    "dense_misaligned": dict(n0=32768, hot=hot_dense, layout=lambda: amp.dense(32768), x_off=1),
    "causal": dict(n0=16384, hot=lambda r: hot_causal(r)[0], layout=lambda: amp.causal(1, 128, 128)),
    # weight kernel (a weight shared by the 8 samples), one scale per tensor / per output channel
    "weight": dict(n0=32768, hot=hot_dense, linear=True),
    "weight_rows": dict(n0=32768, hot=hot_dense, linear=True, row_len=4096),
    # streaming kernels with one scale per row
    "rows_long": dict(n0=32768, hot=hot_dense, layout=lambda: amp.dense(32768, 4096), row_len=4096),
    "rows_causal": dict(n0=16384, hot=lambda r: hot_causal(r)[0], layout=lambda: amp.causal(1, 128, 128),
                        row_len=128),
    "rows_short": dict(n0=32768, hot=hot_dense, layout=lambda: amp.dense(32768, 128), row_len=128),
    "rows_24": dict(n0=24 * 1366, hot=hot_dense, layout=lambda: amp.dense(24 * 1366, 24), row_len=24),
    "rows_20": dict(n0=20 * 1639, hot=hot_dense, layout=lambda: amp.dense(20 * 1639, 20), row_len=20),
    # the single-read pass: row scales computed by the pass itself from each row's absmax
    "single_read_512": dict(n0=32768, hot=hot_dense, layout=lambda: amp.dense(32768, 512), row_len=512, computed=True),
    "single_read_128": dict(n0=32768, hot=hot_dense, layout=lambda: amp.dense(32768, 128), row_len=128, computed=True),
    "single_read_11008": dict(n0=11008 * 3, hot=hot_dense, layout=lambda: amp.dense(11008 * 3, 11008), row_len=11008,
                              computed=True),
    "single_read_causal": dict(n0=16384, hot=lambda r: hot_causal(r)[0], layout=lambda: amp.causal(1, 128, 128),
                               row_len=128, computed=True),
    # the same with the power-of-two rule: scales by the rule from each row's absmax, cast by the scaled conversions
    "single_read_512_pow2": dict(n0=32768, hot=hot_dense, layout=lambda: amp.dense(32768, 512), row_len=512,
                                 computed=True, pow2_rule=True),
    "single_read_causal_pow2": dict(n0=16384, hot=lambda r: hot_causal(r)[0], layout=lambda: amp.causal(1, 128, 128),
                                    row_len=128, computed=True, pow2_rule=True),
}
# paths with one scale per tensor that have a scaled-conversion variant (streaming kernel)
POW2_PATHS = ["dense", "dense_misaligned", "causal"]


def run_path(path, rng_name):
    P = PATHS[path]
    rg = RANGES_POW2[rng_name] if rng_name in RANGES_POW2 else RANGES[rng_name]
    # scaled conversions: the flag on every format of the sensitivity call
    call_fmts = [f | amp.SCALE_POW2 for f in FMTS] if (rng_name in RANGES_POW2 or P.get("pow2_rule")) else FMTS
    n0 = P["n0"]
    x_off = P.get("x_off", 0)
    linear = P.get("linear", False)
    row_len = P.get("row_len")
    computed = P.get("computed", False)
    is_causal = "causal" in path
    nf = len(FMTS)
    pat = patterns_of(rng_name)
    # the pattern buffer, repeated so that every window fits
    need = 8 * N_OPS + x_off + R * n0 + 8
    xbig = np.tile(pat, (need + 65535) // 65536)
    g = f32_to_bf16_bits(G_BASE * np.float32(2.0 ** rg["gexp"]))
    hot = [P["hot"](r) for r in range(R)]
    z = np.zeros((R, n0), dtype=np.uint16)
    for r in range(R):
        z[r, hot[r]] = g[r]
    X, Z = dev_bits(xbig), dev_bits(z.reshape(-1))
    sc = scales_of(rng_name)
    rows_per_sample = 0
    if row_len:
        # one scale per row, rows differ; the table is shared by all ops
        rows_per_sample = n0 // row_len
        n_rows = rows_per_sample * (1 if linear else R)
        mult = ROW_MULT[np.arange(n_rows) % 8]
        t_scale = np.stack([np.float32(sc[f][0]) * mult for f in range(nf)], axis=1).astype(np.float32)
        t_inv = np.stack([np.float32(sc[f][1]) / mult for f in range(nf)], axis=1).astype(np.float32)
    else:
        t_scale = np.array([[sc[f][0] for f in range(nf)]], dtype=np.float32)
        t_inv = np.array([[sc[f][1] for f in range(nf)]], dtype=np.float32)
    S, I = torch.from_numpy(t_scale).to(DEV), torch.from_numpy(t_inv).to(DEV)

    xb, zb, sb, ib = X.data_ptr(), Z.data_ptr(), S.data_ptr(), I.data_ptr()
    ops = []
    for k in range(N_OPS):
        if linear:
            d = amp.LinearDesc()
            d.w, d.dw = xb + 2 * (8 * k), zb
            d.C, d.K, d.tokens, d.R = 4096, n0 // 4096, 0, R
            d.w_scale, d.w_inv = sb, ib
            d.scale_rows = amp.ROWS_OPERAND1 if row_len else 0
        else:
            d = amp.BgemmDesc()
            d.x0, d.dx0 = xb + 2 * (8 * k + x_off), zb
            d.layout0, d.layout1, d.R = P["layout"](), amp.dense(0), R
            d.scale0, d.inv0 = sb, ib
            d.scale_rows = (amp.ROWS_COMPUTE0 if computed else amp.ROWS_OPERAND0) if row_len else 0
        ops.append(d)
    out = torch.full((N_OPS * R, nf, 4), -1.0, dtype=torch.float32, device=DEV)
    if linear:
        ws = torch.empty(amp.amp_sens_linear_workspace_bytes(ops, nf), dtype=torch.uint8, device=DEV)
        amp.amp_sens_linear(ops, call_fmts, out, ws)
    else:
        ws = torch.empty(amp.amp_sens_bgemm_workspace_bytes(ops, nf), dtype=torch.uint8, device=DEV)
        amp.amp_sens_bgemm(ops, call_fmts, out, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy().reshape(N_OPS, R, nf, 4)
    col = 2 if linear else 0

    seen = np.zeros(65536, dtype=bool)
    ks = np.arange(N_OPS)
    for r in range(R):
        idx = (8 * ks + x_off + (0 if linear else r * n0) + hot[r]) % 65536
        seen[idx] = True
        xs = pat[idx]
        row = 0
        if row_len:
            in_sample = hot_causal(r)[1] if is_causal else hot[r] // row_len
            row = (0 if linear else r * rows_per_sample) + in_sample
        if computed:
            # the scales are those of the hot element's row, which differs from op to op: gather every
            # op's row (its valid part) and let the oracle derive its scales
            valid = hot_causal(r)[1] + 1 if is_causal else row_len
            start = 8 * ks + x_off + r * n0 + in_sample * row_len
            rows_x = xbig[start[:, None] + np.arange(valid)[None, :]]
        for fi, f in enumerate(FMTS):
            if computed:
                am_k, sc_k, iv_k, _ = oracle.absmax_scale_rows(rows_x.reshape(-1), N_OPS, valid, f)
                if P.get("pow2_rule"):
                    both = [oracle.scale_pow2(int(b), f) for b in (parity.bits32(am_k) >> 16)]
                    sc_k = np.array([b_[0] for b_ in both], dtype=np.float32)
                    iv_k = np.array([b_[1] for b_ in both], dtype=np.float32)
                E, A = np.empty(N_OPS), np.empty(N_OPS)
                pairs_of = {}
                for k in range(N_OPS):
                    pairs_of.setdefault((sc_k[k].tobytes(), iv_k[k].tobytes()), []).append(k)
                for ids in pairs_of.values():
                    ids = np.array(ids)
                    e_, a_ = oracle.sens_operand(xs[ids], np.full(ids.size, g[r], dtype=np.uint16), ids.size, 1,
                                                 sc_k[ids[0]], iv_k[ids[0]], f)
                    E[ids], A[ids] = e_, a_
            else:
                E, A = oracle.sens_operand(xs, np.full(N_OPS, g[r], dtype=np.uint16), N_OPS, 1, t_scale[row, fi], t_inv[row, fi], f)
            tag = "%s %s sample %d fmt %d" % (path, rng_name, r, f)
            parity.assert_sum_close(got[:, r, fi, col + 1], A, 0.0, tag + " A")
            # with scales derived from the row, an element next to the grid has an error far below the
            # value itself, whose square can leave the normal fp32 range: no relative claim down there
            parity.assert_sum_close(got[:, r, fi, col], E, 1e-36 if computed else 0.0, tag + " E")
            other = got[:, r, fi, 0:2] if linear else got[:, r, fi, 2:]
            assert np.all(other == 0), tag + ": the empty operand"
    assert seen.all(), "the sweep must visit every pattern"


@pytest.mark.parametrize("rng_name", list(RANGES))
@pytest.mark.parametrize("path", list(PATHS))
def test_every_pattern_through_a_fused_kernel(path, rng_name):
    say("pattern sweep through %s, value range %s" % (path, rng_name))
    run_path(path, rng_name)


@pytest.mark.parametrize("rng_name", list(RANGES_POW2))
@pytest.mark.parametrize("path", POW2_PATHS)
def test_every_pattern_through_the_scaled_conversions(path, rng_name):
    say("pattern sweep through %s with the scaled conversions, value range %s" % (path, rng_name))
    run_path(path, rng_name)
