"""Pins for the oracle's absmax/scale, the two sums E and A, and the epilogue.

No GPU, no GPU library.  Pins: hand-worked cases (tests/golden/sens_hand_case.txt), an
fp64 library dot product for A, exact rational closed forms for the rounding error of
uniform mantissas, the bounds that follow from half-ulp rounding, additivity and
masking identities, and the constants the paper prints (alpha_f, Sec. 2.2).
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from helpers import bf16_bits_to_f64, f32_to_bf16_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sens_hand_case.txt")
FMAX = {oracle.E4M3: 448.0, oracle.E5M2: 57344.0}
MBITS = {oracle.E4M3: 3, oracle.E5M2: 2}


def hand_cases():
    cases = {}
    for line in open(GOLDEN):
        tok = line.split("#")[0].split()
        if not tok:
            continue
        c = cases.setdefault(tok[0], {})
        if tok[1] == "scale":
            c["scale"], c["inv"] = float(tok[2]), float(tok[4])
        elif tok[1] in ("x", "xdot"):
            c[tok[1]] = np.array([float(t) for t in tok[2:]], dtype=np.float32)
        else:
            c[tok[1]] = float(tok[2])
    return cases


@pytest.mark.parametrize("name", ["case1", "case2"])
def test_hand_worked_sums(name):
    c = hand_cases()[name]
    x, g = f32_to_bf16_bits(c["x"]), f32_to_bf16_bits(c["xdot"])
    assert np.array_equal(bf16_bits_to_f64(x), c["x"].astype(np.float64))   # inputs are bf16-exact
    E, A = oracle.sens_operand(x, g, 1, x.size, c["scale"], c["inv"], oracle.E4M3)
    assert E[0] == c["E"]
    assert A[0] == c["A"]


def test_alpha_constants():
    # alpha_f = 2^(-2 m_f)/12: 1/768 for three mantissa bits, 1/192 for two
    assert oracle.alpha(3) == 1.0 / 768.0
    assert oracle.alpha(2) == 1.0 / 192.0
    assert oracle.alpha(0) == 1.0 / 12.0


def rand_bf16(rng, n, sigma=1.0):
    return f32_to_bf16_bits((rng.standard_normal(n) * sigma).astype(np.float32))


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_A_is_squared_norm_of_elementwise_product(fmt):
    rng = np.random.default_rng(3)
    R, n = 3, 5001
    x, g = rand_bf16(rng, R * n), rand_bf16(rng, R * n, 1e-3)
    am, sc, iv, fl = oracle.absmax_scale(x, fmt)
    E, A = oracle.sens_operand(x, g, R, n, sc, iv, fmt)
    xv, gv = bf16_bits_to_f64(x).reshape(R, n), bf16_bits_to_f64(g).reshape(R, n)
    for r in range(R):
        t = xv[r] * gv[r]
        assert A[r] == pytest.approx(np.dot(t, t), rel=1e-13)
    # xdot == 1 -> A = ||x||^2 ; xdot == c -> E scales by c^2
    ones = f32_to_bf16_bits(np.ones(R * n, dtype=np.float32))
    E1, A1 = oracle.sens_operand(x, ones, R, n, sc, iv, fmt)
    assert A1[0] == pytest.approx(np.dot(xv[0], xv[0]), rel=1e-13)
    fours = f32_to_bf16_bits(np.full(R * n, 4.0, dtype=np.float32))
    E4, A4 = oracle.sens_operand(x, fours, R, n, sc, iv, fmt)
    assert np.allclose(E4, 16.0 * E1, rtol=1e-14) and np.allclose(A4, 16.0 * A1, rtol=1e-14)


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_E_equals_error_of_dequantised_tensor(fmt):
    """E recomputed from the oracle's own codes via the pinned decode table (ties the sum to
    the separately pinned cast) and checked against the half-ulp bound."""
    rng = np.random.default_rng(11)
    n = 20000
    x, g = rand_bf16(rng, n), rand_bf16(rng, n, 1e-3)
    am, sc, iv, fl = oracle.absmax_scale(x, fmt)
    codes, deq = oracle.fake_quant_fp8(x, sc, iv, fmt)
    q = oracle.fp8_decode_table(fmt)[codes]
    xv, gv = bf16_bits_to_f64(x), bf16_bits_to_f64(g)
    e = xv - q * np.float64(sc)
    E, A = oracle.sens_operand(x, g, 1, n, sc, iv, fmt)
    assert E[0] == pytest.approx(np.sum((gv * e) ** 2), rel=1e-13)
    # dequant is one fp32 multiply of q by scale
    assert np.array_equal(deq, (q.astype(np.float32) * np.float32(sc)))


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
@pytest.mark.parametrize("exp", [-3, 0, 5])
def test_closed_form_uniform_mantissas(fmt, exp):
    """All 128 bf16 mantissas of one normal binade, scale 1, xdot = 1:
    mean(e^2)/ulp^2 = (1 + 2/n^2)/12 exactly, n = 2^(7-m) inputs per FP8 interval."""
    m = MBITS[fmt]
    n_per = 2 ** (7 - m)
    xs = [Fraction(2) ** exp * (1 + Fraction(k, 128)) for k in range(128)]
    x = f32_to_bf16_bits(np.array([float(v) for v in xs], dtype=np.float32))
    ones = f32_to_bf16_bits(np.ones(128, dtype=np.float32))
    E, A = oracle.sens_operand(x, ones, 1, 128, 1.0, 1.0, fmt)
    ulp = Fraction(2) ** (exp - m)
    want_E = 128 * ulp ** 2 * (1 + Fraction(2, n_per ** 2)) / 12
    want_A = sum(v * v for v in xs)
    assert E[0] == pytest.approx(float(want_E), rel=1e-15)
    assert A[0] == pytest.approx(float(want_A), rel=1e-15)
    ratio = (E[0] / A[0]) / oracle.alpha(m)
    assert ratio == pytest.approx(0.4341 if fmt == oracle.E4M3 else 0.4316, abs=5e-4)


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_noise_model_envelope_on_random_mantissas(fmt):
    """Random uniform mantissas over many normal binades: the measured E/A sits near the
    3/7-type constant of the closed form and inside (alpha/4, alpha]; hard bound E <= 3 alpha A."""
    rng = np.random.default_rng(5)
    n = 400000
    m = MBITS[fmt]
    lo = -4 if fmt == oracle.E4M3 else -12
    mant = 1.0 + rng.integers(0, 128, n) / 128.0
    x = f32_to_bf16_bits((mant * np.exp2(rng.integers(lo, 8, n)) * rng.choice([-1, 1], n)).astype(np.float32))
    g = f32_to_bf16_bits(np.exp(rng.normal(0, 0.5, n)).astype(np.float32))
    E, A = oracle.sens_operand(x, g, 1, n, 1.0, 1.0, fmt)
    ratio = E[0] / A[0] / oracle.alpha(m)
    assert 0.25 < ratio <= 1.0
    assert ratio == pytest.approx(0.4341 if fmt == oracle.E4M3 else 0.4316, rel=0.02)
    assert E[0] <= 3 * oracle.alpha(m) * A[0]


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_zero_error_on_grid_values_at_scale_one(fmt):
    t = oracle.fp8_decode_table(fmt)
    grid = t[np.isfinite(t)].astype(np.float32)
    x = f32_to_bf16_bits(grid)
    assert np.array_equal(bf16_bits_to_f64(x), grid.astype(np.float64))     # grid fits bf16
    g = f32_to_bf16_bits(np.full(grid.size, 3.0, dtype=np.float32))
    E, A = oracle.sens_operand(x, g, 1, grid.size, 1.0, 1.0, fmt)
    assert E[0] == 0.0 and A[0] > 0.0


def test_additive_over_concatenation_and_permutation():
    rng = np.random.default_rng(9)
    n = 4096
    x, g = rand_bf16(rng, 2 * n), rand_bf16(rng, 2 * n, 1e-3)
    sc, iv = np.float32(0.013), np.float32(1 / 0.013)
    E, A = oracle.sens_operand(x, g, 1, 2 * n, sc, iv, oracle.E4M3)
    Eh, Ah = oracle.sens_operand(x, g, 2, n, sc, iv, oracle.E4M3)      # same data as two samples
    assert E[0] == pytest.approx(Eh.sum(), rel=1e-13) and A[0] == pytest.approx(Ah.sum(), rel=1e-13)
    p = rng.permutation(2 * n)
    Ep, Ap = oracle.sens_operand(x[p], g[p], 1, 2 * n, sc, iv, oracle.E4M3)
    assert E[0] == pytest.approx(Ep[0], rel=1e-12) and A[0] == pytest.approx(Ap[0], rel=1e-12)


@pytest.mark.parametrize("rows,cols", [(8, 8), (5, 9), (7, 3), (16, 24)])
def test_causal_equals_dense_with_explicit_zeros(rows, cols):
    rng = np.random.default_rng(rows * 100 + cols)
    R, batch = 2, 3
    n = batch * rows * cols
    x, g = rand_bf16(rng, R * n), rand_bf16(rng, R * n)
    i = np.arange(rows)[:, None]
    j = np.arange(cols)[None, :]
    keep = (j <= i + (cols - rows))
    mask = np.broadcast_to(keep, (R, batch, rows, cols)).reshape(-1)
    xz, gz = np.where(mask, x, 0).astype(np.uint16), np.where(mask, g, 0).astype(np.uint16)
    sc, iv = np.float32(0.01), np.float32(100.0)
    Ec, Ac = oracle.sens_operand(x, g, R, 0, sc, iv, oracle.E4M3, causal=(batch, rows, cols))
    Ed, Ad = oracle.sens_operand(xz, gz, R, n, sc, iv, oracle.E4M3)
    assert np.array_equal(Ec, Ed) and np.array_equal(Ac, Ad)
    # absmax over a causal operand ignores the masked entries
    big = x.copy()
    big[~mask] = f32_to_bf16_bits(np.array([1e6], dtype=np.float32))[0]
    am_c = oracle.absmax_scale(big, oracle.E4M3, causal=(batch, rows, cols))[0]
    am_d = oracle.absmax_scale(xz, oracle.E4M3)[0]
    assert am_c == am_d


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_absmax_scale_pins(fmt):
    F = np.float32(FMAX[fmt])
    x = f32_to_bf16_bits(np.array([0.5, -3.0, 2.0, float(F)], dtype=np.float32))
    am, sc, iv, fl = oracle.absmax_scale(x, fmt)
    assert (am, sc, iv, fl) == (F, 1.0, 1.0, 0)                      # amax = FMAX -> unit scale
    x = f32_to_bf16_bits(np.array([0.5, -3.0, 2.0], dtype=np.float32))
    am, sc, iv, fl = oracle.absmax_scale(x, fmt)
    assert am == 3.0 and sc == np.float32(3.0) / F and iv == F / np.float32(3.0) and fl == 0
    assert abs(float(sc) * float(F) - 3.0) <= 3.0 * 2.0 ** -23
    zeros = np.zeros(7, dtype=np.uint16)
    zeros[3] = 0x8000
    assert oracle.absmax_scale(zeros, fmt) == (0.0, 1.0, 1.0, 0)
    tiny = np.array([0x0001], dtype=np.uint16)                      # bf16 subnormal 2^-133
    am, sc, iv, fl = oracle.absmax_scale(tiny, fmt)
    assert am == np.float32(2.0 ** -133) and (sc, iv) == (1.0, 1.0)  # reciprocal would overflow
    inf = np.array([0x3F80, 0xFF80], dtype=np.uint16)
    assert oracle.absmax_scale(inf, fmt)[3] == 1
    nan = np.array([0x3F80, 0x7FC0], dtype=np.uint16)
    assert oracle.absmax_scale(nan, fmt)[3] == 1
    # the largest element maps onto the largest code (the clamp absorbs a 1-ulp overshoot)
    rng = np.random.default_rng(1)
    for _ in range(50):
        x = rand_bf16(rng, 64, float(np.exp(rng.normal(0, 3))))
        am, sc, iv, fl = oracle.absmax_scale(x, fmt)
        codes, _ = oracle.fake_quant_fp8(x, sc, iv, fmt)
        k = np.argmax(np.abs(bf16_bits_to_f64(x)))
        assert codes[k] & 0x7F == (0x7E if fmt == oracle.E4M3 else 0x7B)


def test_linear_and_bgemm_wrappers_compose_operands():
    rng = np.random.default_rng(21)
    R, Cd, K = 3, 24, 10
    row_off = np.array([0, 5, 6, 13], dtype=np.int64)               # ragged samples
    x, dx = rand_bf16(rng, 13 * Cd), rand_bf16(rng, 13 * Cd, 1e-3)
    w, dw = rand_bf16(rng, K * Cd, 0.02), rand_bf16(rng, R * K * Cd, 1e-3)
    _, xs, xi, _ = oracle.absmax_scale(x, oracle.E5M2)
    _, ws, wi, _ = oracle.absmax_scale(w, oracle.E5M2)
    out = oracle.sens_linear(x, dx, w, dw, Cd, K, R, row_off, xs, xi, ws, wi, oracle.E5M2)
    for r in range(R):
        a, b = row_off[r] * Cd, row_off[r + 1] * Cd
        E, A = oracle.sens_operand(x[a:b], dx[a:b], 1, b - a, xs, xi, oracle.E5M2)
        assert (out[r, 0], out[r, 1]) == (E[0], A[0])
    Ew, Aw = oracle.sens_operand(w, dw, R, K * Cd, ws, wi, oracle.E5M2, x_shared=True)
    assert np.array_equal(out[:, 2], Ew) and np.array_equal(out[:, 3], Aw)

    H, S, D = 2, 8, 4
    p, dp = rand_bf16(rng, R * H * S * S), rand_bf16(rng, R * H * S * S, 1e-3)
    v, dv = rand_bf16(rng, R * H * S * D), rand_bf16(rng, R * H * S * D, 1e-3)
    out = oracle.sens_bgemm(p, dp, ("causal", H, S, S), v, dv, ("dense", H * S * D), R,
                            0.01, 100.0, 0.02, 50.0, oracle.E4M3)
    E0, A0 = oracle.sens_operand(p, dp, R, 0, 0.01, 100.0, oracle.E4M3, causal=(H, S, S))
    E1, A1 = oracle.sens_operand(v, dv, R, H * S * D, 0.02, 50.0, oracle.E4M3)
    assert np.array_equal(out, np.stack([E0, A0, E1, A1], axis=1))


def test_epilogue_mean_sensitivity_and_group_mse():
    # s_l = mean_r (A_0^r + A_1^r); d_{l,f} = s_l alpha_f; d_{j,p} additive over a group's layers
    A0, A1 = np.array([1.0, 2.0, 6.0]), np.array([0.5, 0.25, 0.25])
    assert oracle.layer_sensitivity(A0, A1) == pytest.approx(10.0 / 3.0, rel=1e-15)
    s = np.array([2.0, 3.0, 5.0])
    alphas = np.array([0.0, 1.0 / 768.0, 1.0 / 192.0])              # BF16, E4M3, E5M2
    d = oracle.group_mse(s, alphas)
    assert d.size == 27 and d[0] == 0.0
    for p in range(27):
        digits = [(p // 3 ** l) % 3 for l in range(3)]
        assert d[p] == pytest.approx(sum(s[l] * alphas[digits[l]] for l in range(3)), rel=1e-15)
    assert d[26] == pytest.approx(10.0 / 192.0, rel=1e-15)


# ---- one scale per row ---------------------------------------------------------------------------

def rows_hand_case():
    c = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "sens_rows_hand_case.txt")):
        tok = line.split("#")[0].split()
        if tok:
            c[tok[0]] = [float(t) for t in tok[1:]]
    return c


def test_rows_hand_worked_sums():
    c = rows_hand_case()
    n_rows, row_len = int(c["rows"][0]), int(c["rows"][1])
    x = f32_to_bf16_bits(np.array(c["x"], dtype=np.float32))
    g = f32_to_bf16_bits(np.array(c["xdot"], dtype=np.float32))
    assert np.array_equal(bf16_bits_to_f64(x), np.array(c["x"]))
    E, A = oracle.sens_operand_rows(x, g, n_rows, row_len, c["scale"], c["inv"], oracle.E4M3)
    assert E == c["E"][0] and A == c["A"][0]
    # a row paired with the other row's scale is a different, also hand-worked, number
    E2, A2 = oracle.sens_operand_rows(x, g, n_rows, row_len, c["scale"][::-1], c["inv"][::-1], oracle.E4M3)
    assert E2 == c["E_exchanged"][0] and A2 == c["A"][0]


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_rows_with_one_common_scale_is_the_per_tensor_sum(fmt):
    rng = np.random.default_rng(11)
    n_rows, row_len = 7, 53
    x, g = rand_bf16(rng, n_rows * row_len), rand_bf16(rng, n_rows * row_len, 1e-2)
    am, sc, iv, fl = oracle.absmax_scale(x, fmt)
    E, A = oracle.sens_operand(x, g, 1, x.size, sc, iv, fmt)
    Er, Ar = oracle.sens_operand_rows(x, g, n_rows, row_len, np.full(n_rows, sc), np.full(n_rows, iv), fmt)
    assert Er == pytest.approx(E[0], rel=1e-14) and Ar == pytest.approx(A[0], rel=1e-14)


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_rows_is_the_sum_over_rows_each_cast_as_its_own_tensor(fmt):
    rng = np.random.default_rng(12)
    n_rows, row_len = 9, 40
    x = f32_to_bf16_bits((rng.standard_normal((n_rows, row_len)) *
                          np.exp(rng.normal(0, 2, (n_rows, 1)))).astype(np.float32)).reshape(-1)
    g = rand_bf16(rng, n_rows * row_len, 1e-2)
    am, sc, iv, fl = oracle.absmax_scale_rows(x, n_rows, row_len, fmt)
    xv = np.abs(bf16_bits_to_f64(x)).reshape(n_rows, row_len)
    assert np.array_equal(am.astype(np.float64), xv.max(axis=1))
    assert fl == 0
    E = A = 0.0
    for i in range(n_rows):
        xi, gi = x[i * row_len:(i + 1) * row_len], g[i * row_len:(i + 1) * row_len]
        a1, s1, i1, _ = oracle.absmax_scale(xi, fmt)
        assert (a1, s1, i1) == (am[i], sc[i], iv[i])
        e, a = oracle.sens_operand(xi, gi, 1, row_len, s1, i1, fmt)
        E, A = E + e[0], A + a[0]
    Er, Ar = oracle.sens_operand_rows(x, g, n_rows, row_len, sc, iv, fmt)
    assert Er == pytest.approx(E, rel=1e-13) and Ar == pytest.approx(A, rel=1e-13)


def test_rows_causal_rows_own_their_prefix_only():
    rng = np.random.default_rng(13)
    mats, rows, cols = 3, 5, 7                               # row i owns i + 3 entries
    x = rand_bf16(rng, mats * rows * cols).reshape(mats, rows, cols)
    g = rand_bf16(rng, mats * rows * cols, 1e-2).reshape(mats, rows, cols)
    big = f32_to_bf16_bits(np.array([3e38], dtype=np.float32))[0]
    lens = [min(cols, i + 1 + cols - rows) for i in range(rows)]
    for i in range(rows):
        x[:, i, lens[i]:] = big                              # junk outside the operand
        g[:, i, lens[i]:] = big
    fmt = oracle.E4M3
    am, sc, iv, fl = oracle.absmax_scale_rows(x.reshape(-1), mats * rows, cols, fmt, causal_rows=rows)
    assert fl == 0 and float(am.max()) < 10.0
    E = A = 0.0
    for m in range(mats):
        for i in range(rows):
            xi, gi = x[m, i, :lens[i]].copy(), g[m, i, :lens[i]].copy()
            a1, s1, i1, _ = oracle.absmax_scale(xi, fmt)
            assert (a1, s1, i1) == (am[m * rows + i], sc[m * rows + i], iv[m * rows + i])
            e, a = oracle.sens_operand(xi, gi, 1, lens[i], s1, i1, fmt)
            E, A = E + e[0], A + a[0]
    Er, Ar = oracle.sens_operand_rows(x.reshape(-1), g.reshape(-1), mats * rows, cols, sc, iv, fmt, causal_rows=rows)
    assert Er == pytest.approx(E, rel=1e-13) and Ar == pytest.approx(A, rel=1e-13)


def test_rows_scale_removes_the_error_a_loud_row_causes_in_quiet_rows():
    """Why finer granularity matters: with one scale for the tensor a row of large values pushes
    the small rows into the subnormal range of the format; with a scale per row every row keeps
    the relative accuracy of reading 6 (E <= 3 alpha A)."""
    rng = np.random.default_rng(14)
    n_rows, row_len = 4, 256
    xv = rng.standard_normal((n_rows, row_len)).astype(np.float32)
    xv[0] *= 2.0 ** 18
    x = f32_to_bf16_bits(xv).reshape(-1)
    g = f32_to_bf16_bits(np.ones(n_rows * row_len, dtype=np.float32))
    fmt = oracle.E4M3
    am, sc, iv, _ = oracle.absmax_scale(x, fmt)
    Et, At = oracle.sens_operand(x[row_len:], g[row_len:], 1, 3 * row_len, sc, iv, fmt)
    amr, scr, ivr, _ = oracle.absmax_scale_rows(x, n_rows, row_len, fmt)
    Er, Ar = oracle.sens_operand_rows(x[row_len:], g[row_len:], 3, row_len, scr[1:], ivr[1:], fmt)
    assert Ar == pytest.approx(At[0], rel=1e-14)
    assert Er <= 3 * oracle.alpha(3) * Ar
    assert Et[0] > 20 * Er


# ---- power-of-two scales ---------------------------------------------------------------------------

@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_pow2_scale_is_the_smallest_power_of_two_that_fits(fmt):
    from fractions import Fraction
    fmax = Fraction(int(FMAX[fmt]))
    pats = np.concatenate([np.arange(1, 0x7F80, 37, dtype=np.uint16),           # spread over all magnitudes
                           np.array([1, 2, 0x007F, 0x0080, 0x0081, 0x7F7F], dtype=np.uint16)])
    # amax = FMAX * 2^k exactly, and its bf16 neighbours
    exact = f32_to_bf16_bits(np.array([FMAX[fmt] * 2.0 ** k for k in range(-100, 100, 7)], dtype=np.float32))
    pats = np.concatenate([pats, exact, exact + 1, exact - 1]).astype(np.uint16)
    vals = bf16_bits_to_f64(pats)
    for h, v in zip(pats, vals):
        sc, iv = oracle.scale_pow2(h, fmt)
        a = Fraction(float(v))
        s = Fraction(float(sc))
        if sc == 1.0 and iv == 1.0 and not (a / 1 <= fmax and a * 2 > fmax):
            # fallback: only where 1 / s is not an fp32 number
            k_true = 0
            while fmax * Fraction(2) ** k_true < a:
                k_true += 1
            while fmax * Fraction(2) ** (k_true - 1) >= a:
                k_true -= 1
            assert k_true < -126 or k_true > 127, (h, v)
            continue
        assert s.numerator == 1 or s.denominator == 1                             # a power of two ...
        assert (s.numerator & (s.numerator - 1)) == 0 and (s.denominator & (s.denominator - 1)) == 0
        assert a / s <= fmax and a / (s / 2) > fmax                                # ... the smallest that fits
        assert Fraction(float(iv)) * s == 1
    assert oracle.scale_pow2(0, fmt) == (1.0, 1.0)
    sc, iv = oracle.scale_pow2(f32_to_bf16_bits(np.array([FMAX[fmt] * 4], dtype=np.float32))[0], fmt)
    assert (sc, iv) == (4.0, 0.25)


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_pow2_scale_commutes_with_the_cast(fmt):
    """At a power-of-two scale s the cast of x is the cast of x / s at scale 1, so E(x; s) = s^2 E(x / s; 1)
    exactly, and values on the grid times s have zero error."""
    rng = np.random.default_rng(21)
    x = rand_bf16(rng, 4000, 3.0)
    g = f32_to_bf16_bits(np.ones(4000, dtype=np.float32))
    am = np.abs(bf16_bits_to_f64(x)).max()
    amax_bits = f32_to_bf16_bits(np.array([am], dtype=np.float32))[0]
    sc, iv = oracle.scale_pow2(amax_bits, fmt)
    assert sc != 1.0
    xs = f32_to_bf16_bits((bf16_bits_to_f64(x) * float(iv)).astype(np.float32))    # exact: power of two
    E, A = oracle.sens_operand(x, g, 1, x.size, sc, iv, fmt)
    E1, A1 = oracle.sens_operand(xs, g, 1, x.size, 1.0, 1.0, fmt)
    assert E[0] == pytest.approx(float(sc) ** 2 * E1[0], rel=1e-15)
    codes, deq = oracle.fake_quant_fp8(x, sc, iv, fmt)
    on_grid = f32_to_bf16_bits(deq)
    assert np.array_equal(bf16_bits_to_f64(on_grid), deq.astype(np.float64))        # FP8 values times 2^k are bf16
    E0, _ = oracle.sens_operand(on_grid, g, 1, x.size, sc, iv, fmt)
    assert E0[0] == 0.0


# ---- one scale per 1 x B block of a row ----------------------------------------------------------

def blocks_hand_case():
    c = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "sens_blocks_hand_case.txt")):
        tok = line.split("#")[0].split()
        if tok:
            c[tok[0]] = [float(t) for t in tok[1:]]
    return c


def test_blocks_hand_worked_sums_and_absmax():
    c = blocks_hand_case()
    n_rows, row_len, B = int(c["rows"][0]), int(c["rows"][1]), int(c["block"][0])
    x = f32_to_bf16_bits(np.array(c["x"], dtype=np.float32))
    g = f32_to_bf16_bits(np.array(c["xdot"], dtype=np.float32))
    assert np.array_equal(bf16_bits_to_f64(x), np.array(c["x"]))
    assert np.array_equal(bf16_bits_to_f64(g), np.array(c["xdot"]))
    E, A = oracle.sens_operand_blocks(x, g, n_rows, row_len, B, c["scale"], c["inv"], oracle.E4M3)
    assert E == c["E"][0] and A == c["A"][0]
    # any other assignment of the four scales to the four blocks makes some value saturate: a different E
    import itertools
    for perm in itertools.permutations(range(4)):
        if perm == (0, 1, 2, 3):
            continue
        sc = [c["scale"][p] for p in perm]
        iv = [c["inv"][p] for p in perm]
        E2, A2 = oracle.sens_operand_blocks(x, g, n_rows, row_len, B, sc, iv, oracle.E4M3)
        assert E2 != c["E"][0] and A2 == c["A"][0], perm
    am, sc, iv, fl = oracle.absmax_scale_blocks(x, n_rows, row_len, B, oracle.E4M3)
    assert fl == 0 and np.array_equal(am.reshape(-1).astype(np.float64), np.array(c["amax"]))
    want = np.array(c["amax"], dtype=np.float32)
    assert np.array_equal(sc.reshape(-1), want / np.float32(448.0))      # numpy's fp32 division, not the oracle's
    assert np.array_equal(iv.reshape(-1), np.float32(448.0) / want)


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_blocks_are_the_rows_of_the_operand_reshaped(fmt):
    """[n_rows, row_len] cut into 1 x B blocks is the same set of scale groups as [n_rows * row_len / B, B]
    with one scale per row; a block as long as the row is one scale per row; one common scale is the
    per-tensor sum."""
    rng = np.random.default_rng(21)
    n_rows, row_len, B = 6, 48, 16
    x = f32_to_bf16_bits((rng.standard_normal((n_rows, row_len // B, B)) *
                          np.exp(rng.normal(0, 2, (n_rows, row_len // B, 1)))).astype(np.float32)).reshape(-1)
    g = rand_bf16(rng, n_rows * row_len, 1e-2)
    am, sc, iv, fl = oracle.absmax_scale_blocks(x, n_rows, row_len, B, fmt)
    am_r, sc_r, iv_r, _ = oracle.absmax_scale_rows(x, n_rows * row_len // B, B, fmt)
    assert np.array_equal(am.reshape(-1), am_r) and np.array_equal(sc.reshape(-1), sc_r) and np.array_equal(iv.reshape(-1), iv_r)
    E, A = oracle.sens_operand_blocks(x, g, n_rows, row_len, B, sc, iv, fmt)
    Er, Ar = oracle.sens_operand_rows(x, g, n_rows * row_len // B, B, sc_r, iv_r, fmt)
    assert E == pytest.approx(Er, rel=1e-13) and A == pytest.approx(Ar, rel=1e-13)
    # B = row_len
    am1, sc1, iv1, _ = oracle.absmax_scale_blocks(x, n_rows, row_len, row_len, fmt)
    am2, sc2, iv2, _ = oracle.absmax_scale_rows(x, n_rows, row_len, fmt)
    assert np.array_equal(sc1.reshape(-1), sc2) and np.array_equal(iv1.reshape(-1), iv2) and np.array_equal(am1.reshape(-1), am2)
    E1, A1 = oracle.sens_operand_blocks(x, g, n_rows, row_len, row_len, sc1, iv1, fmt)
    E2, A2 = oracle.sens_operand_rows(x, g, n_rows, row_len, sc2, iv2, fmt)
    assert E1 == pytest.approx(E2, rel=1e-13) and A1 == pytest.approx(A2, rel=1e-13)
    # one scale for all
    a0, s0, i0, _ = oracle.absmax_scale(x, fmt)
    Ec, Ac = oracle.sens_operand_blocks(x, g, n_rows, row_len, B, np.full(sc.shape, s0), np.full(sc.shape, i0), fmt)
    Et, At = oracle.sens_operand(x, g, 1, x.size, s0, i0, fmt)
    assert Ec == pytest.approx(Et[0], rel=1e-13) and Ac == pytest.approx(At[0], rel=1e-13)


def test_blocks_keep_a_loud_channel_from_spoiling_its_row():
    """An outlier channel costs the other blocks of its row nothing: with one scale per block every block
    keeps E <= 3 alpha A (the bound of a normal-range cast), while with one scale per row the quiet blocks
    of a row that holds the outlier lose it."""
    rng = np.random.default_rng(22)
    n_rows, row_len, B = 5, 64, 16
    xf = rng.standard_normal((n_rows, row_len)).astype(np.float32)
    xf[:, 3] *= 1.0e6                                         # the loud channel, in block 0 of every row: the others fall below E4M3's subnormals at its scale
    x = f32_to_bf16_bits(xf).reshape(-1)
    g = f32_to_bf16_bits(np.ones(n_rows * row_len, dtype=np.float32))
    fmt = oracle.E4M3
    alpha = oracle.alpha(oracle.fp8_mantissa_bits(fmt))
    am, sc, iv, _ = oracle.absmax_scale_blocks(x, n_rows, row_len, B, fmt)
    am_r, sc_r, iv_r, _ = oracle.absmax_scale_rows(x, n_rows, row_len, fmt)
    xv = bf16_bits_to_f64(x).reshape(n_rows, row_len)
    for i in range(n_rows):
        for b in range(1, row_len // B):                      # the quiet blocks
            xb = x.reshape(n_rows, row_len)[i, b * B:(b + 1) * B].copy()
            gb = g[:B].copy()
            Eb, Ab = oracle.sens_operand(xb, gb, 1, B, sc[i, b], iv[i, b], fmt)
            assert Eb[0] <= 3 * alpha * Ab[0]
            Er, Ar = oracle.sens_operand(xb, gb, 1, B, sc_r[i], iv_r[i], fmt)
            assert Er[0] > Eb[0]
