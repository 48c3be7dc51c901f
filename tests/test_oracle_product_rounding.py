"""Pin for the one place where the oracle's FP8 code depends on fp32 arithmetic: the product
y = fl32(x * inv) that the cast rounds (scale arithmetic of the library's header; the paper,
Sec. 3.1, leaves the cast unspecified, this is the reading both sides take).

Nothing here calls the oracle to produce an expectation.  For every test pair the exact product is
formed with rational numbers, rounded to fp32 by a rational round-to-nearest-even written here, and
the FP8 code is found by nearest-value search (ties to the even code, saturation) over values
generated here from the OCP format definitions.  The pairs are searched so that the exact product
lies within half an fp32 ulp of a tie between two FP8 values: there the fp32 rounding moves the
product onto the tie (or leaves it off), so an implementation that rounds the exact (or a double)
product straight to FP8, or that fuses the multiply, picks a different code.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle

FORMATS = {oracle.E4M3: dict(ebits=4, mbits=3, bias=7, fmax=448), oracle.E5M2: dict(ebits=5, mbits=2, bias=15, fmax=57344)}


def fp8_values(fmt):
    """[(value as Fraction, code)] of the non-negative finite codes, from the format definition."""
    f = FORMATS[fmt]
    out = []
    for code in range(128):
        e, m = code >> f["mbits"], code & ((1 << f["mbits"]) - 1)
        if e == 0:
            v = Fraction(m, 1 << f["mbits"]) * Fraction(2) ** (1 - f["bias"])
        else:
            v = (1 + Fraction(m, 1 << f["mbits"])) * Fraction(2) ** (e - f["bias"])
        if v <= f["fmax"]:
            out.append((v, code))
    # E4M3 has no infinities and one NaN mantissa; E5M2 keeps the top exponent for inf / NaN
    assert out[-1][0] == f["fmax"]
    return out


def bf16_fraction(bits):
    s, e, m = bits >> 15, (bits >> 7) & 0xFF, bits & 0x7F
    assert e != 0xFF
    v = Fraction(m, 128) * Fraction(2) ** -126 if e == 0 else (1 + Fraction(m, 128)) * Fraction(2) ** (e - 127)
    return -v if s else v


def f32_fraction(x):
    return Fraction(float(np.float32(x)))


def round_to_f32(p):
    """Exact rational -> nearest fp32 (ties to even), as a Fraction; finite range only."""
    if p == 0:
        return Fraction(0)
    s, a = (-1 if p < 0 else 1), abs(p)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    q = Fraction(2) ** (max(e, -126) - 23)               # spacing of fp32 numbers around a
    n = a / q
    k = n.numerator // n.denominator
    r = n - k
    if r > Fraction(1, 2) or (r == Fraction(1, 2) and k % 2 == 1):
        k += 1
    return s * k * q


def nearest_code(y, table, fmax):
    """Code of the FP8 value nearest to the rational y >= 0 (ties to the even code), saturating."""
    if y > fmax:
        y = Fraction(fmax)
    best = None
    for v, code in table:
        d = abs(v - y)
        if best is None or d < best[0] or (d == best[0] and code % 2 == 0 and best[1] % 2 == 1):
            best = (d, code)
    return best[1]


def search_pairs(fmt, rng, per_tie=3):
    """(x bits, inv as np.float32) whose exact product lies within half an fp32 ulp of a tie."""
    table = fp8_values(fmt)
    ties = [(table[i][0] + table[i + 1][0]) / 2 for i in range(len(table) - 1)]
    pairs = []
    for t in ties:
        found = 0
        for _ in range(40):
            if found >= per_tie:
                break
            xb = int(rng.integers(0x3000, 0x4400))                  # 2^-31 .. 2^9, normal bf16
            if rng.random() < 0.5:
                xb |= 0x8000
            x = bf16_fraction(xb)
            inv0 = np.float32(float(t / abs(x)))
            if not np.isfinite(inv0) or inv0 == 0:
                continue
            for step in (0, 1, -1, 2, -2):
                inv = inv0
                for _ in range(abs(step)):
                    inv = np.nextafter(inv, np.float32(np.inf if step > 0 else 0), dtype=np.float32)
                p = abs(x) * f32_fraction(inv)
                ulp = Fraction(2) ** (max(p.numerator.bit_length() - p.denominator.bit_length() - 1, -126) - 23)
                if p != t and abs(p - t) <= ulp / 2 + ulp / 64:
                    pairs.append((xb, np.float32(inv), t))
                    found += 1
                    break
    return table, pairs


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_code_is_decided_by_the_fp32_product(fmt):
    rng = np.random.default_rng(31 + fmt)
    table, pairs = search_pairs(fmt, rng)
    fmax = FORMATS[fmt]["fmax"]
    assert len(pairs) > 150
    on_tie = differs = 0
    for xb, inv, t in pairs:
        x = bf16_fraction(xb)
        p = abs(x) * f32_fraction(inv)
        y = round_to_f32(p)
        want = nearest_code(y, table, fmax) | (0x80 if x < 0 else 0)
        direct = nearest_code(p, table, fmax) | (0x80 if x < 0 else 0)   # what skipping the fp32 rounding gives
        on_tie += y == t
        differs += want != direct
        got, deq = oracle.fake_quant_fp8(np.array([xb], dtype=np.uint16), np.float32(1.0), inv, fmt)
        assert int(got[0]) == want, (hex(xb), float(inv), hex(int(got[0])), hex(want), hex(direct))
        # the same product inside the statistic's routines (each has its own multiply): with
        # xdot = 1 and scale = 1 a one-element operand gives E = (x - q)^2, which names q
        # (neighbouring q differ by an eighth or more; the fp64 subtraction may round)
        q = dict((c, v) for v, c in table)[want & 0x7F] * (-1 if x < 0 else 1)
        e2 = float((x - q) ** 2)
        xa, one = np.array([xb], dtype=np.uint16), np.array([0x3F80], dtype=np.uint16)
        E, A = oracle.sens_operand(xa, one, 1, 1, np.float32(1.0), inv, fmt)
        assert abs(E[0] - e2) <= 1e-14 * e2 and A[0] == float(x * x), (hex(xb), float(inv), E[0], e2)
        Er, Ar = oracle.sens_operand_rows(xa, one, 1, 1, np.array([1.0], np.float32), np.array([inv], np.float32), fmt)
        assert abs(Er - e2) <= 1e-14 * e2 and Ar == float(x * x), (hex(xb), float(inv), Er, e2)
    # the search really produced the discriminating cases
    assert on_tie > 40 and differs > 20, (on_tie, differs)


def test_rational_rounding_helper_against_numpy():
    """round_to_f32 is itself pinned: products of two fp32 numbers computed in float64 are exact
    (48 significant bits), and numpy rounds float64 -> float32 to nearest even."""
    rng = np.random.default_rng(5)
    a = rng.standard_normal(2000).astype(np.float32) * np.float32(3.7)
    b = np.exp(rng.standard_normal(2000) * 8).astype(np.float32)
    for u, v in zip(a, b):
        exact = float(u) * float(v)
        assert round_to_f32(Fraction(float(u)) * Fraction(float(v))) == Fraction(float(np.float32(exact)))
    # subnormal results
    for u, v in ((np.float32(1.1e-20), np.float32(3.3e-21)), (np.float32(2.0 ** -100), np.float32(1.5 * 2.0 ** -49))):
        exact = float(u) * float(v)
        assert round_to_f32(Fraction(float(u)) * Fraction(float(v))) == Fraction(float(np.float32(exact)))
