"""Pins for the oracle's FP8 decode tables and software RNE encoder.

Nothing here calls the GPU library.  The pins are: hand-derived codes from the format
definition (tests/golden/fp8_hand_cases.txt), a library decode/cast (torch's float8
dtypes on the CPU), and brute-force nearest-value search over all 65536 bf16 patterns.
"""
import os

import numpy as np
import pytest
import torch

import oracle
from helpers import all_bf16_patterns, bf16_bits_to_f64, finite_mask

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "fp8_hand_cases.txt")
FMT = {"e4m3": oracle.E4M3, "e5m2": oracle.E5M2}
TORCH8 = {oracle.E4M3: torch.float8_e4m3fn, oracle.E5M2: torch.float8_e5m2}
FMAX = {oracle.E4M3: 448.0, oracle.E5M2: 57344.0}
MBITS = {oracle.E4M3: 3, oracle.E5M2: 2}
EMIN = {oracle.E4M3: -6, oracle.E5M2: -14}


def golden_cases(kind):
    out = []
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if len(line) == 4 and line[0] == kind:
            out.append((FMT[line[1]], float(line[2]), int(line[3], 16)))
    assert out
    return out


@pytest.mark.parametrize("fmt,value,code", golden_cases("decode"))
def test_decode_hand_cases(fmt, value, code):
    assert oracle.fp8_decode_table(fmt)[code] == value


@pytest.mark.parametrize("fmt,value,code", golden_cases("encode"))
def test_encode_hand_cases(fmt, value, code):
    got = oracle.fp8_encode_f32(fmt, np.array([value], dtype=np.float32))[0]
    assert got == code, (hex(got), hex(code))


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_decode_table_structure(fmt):
    t = oracle.fp8_decode_table(fmt)
    finite = np.isfinite(t)
    # E4M3: 256 - 2 NaN; E5M2: 256 - 2 inf - 6 NaN
    assert finite.sum() == (254 if fmt == oracle.E4M3 else 248)
    assert np.isnan(t).sum() == (2 if fmt == oracle.E4M3 else 6)
    assert np.isinf(t).sum() == (0 if fmt == oracle.E4M3 else 2)
    pos = t[:128][finite[:128]]
    assert np.all(np.diff(pos) > 0)                      # strictly increasing in code
    assert pos[0] == 0.0 and pos.max() == FMAX[fmt] == oracle.fp8_max(fmt)
    assert np.array_equal(t[128:][finite[128:]], -pos)   # sign bit mirrors
    assert np.signbit(t[0x80]) and t[0x80] == 0.0
    assert oracle.fp8_mantissa_bits(fmt) == MBITS[fmt]


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_decode_table_matches_library_decode(fmt):
    t = oracle.fp8_decode_table(fmt)
    lib = torch.arange(256, dtype=torch.int32).to(torch.uint8).view(TORCH8[fmt]).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(t), np.isnan(lib))
    ok = ~np.isnan(t)
    assert np.array_equal(t[ok], lib[ok])
    assert np.array_equal(np.signbit(t[ok]), np.signbit(lib[ok]))


def brute_force_codes(fmt, values):
    """Nearest finite table value of the same sign; ties -> even code; beyond max -> max."""
    t = oracle.fp8_decode_table(fmt)
    mags = [(c, t[c]) for c in range(128) if np.isfinite(t[c])]
    codes = np.empty(values.size, dtype=np.uint8)
    tv = np.array([m for _, m in mags])
    tc = np.array([c for c, _ in mags])
    a = np.abs(values)
    a = np.minimum(a, FMAX[fmt])
    for lo in range(0, values.size, 8192):
        blk = a[lo:lo + 8192]
        diff = np.abs(blk[:, None] - tv[None, :])        # exact in fp64
        best = diff.min(axis=1)
        for i in range(blk.size):
            cand = tc[diff[i] == best[i]]
            assert 1 <= cand.size <= 2
            pick = cand[0] if cand.size == 1 else (cand[0] if cand[0] % 2 == 0 else cand[1])
            codes[lo + i] = pick
    codes |= np.where(np.signbit(values), 0x80, 0).astype(np.uint8)
    return codes


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_encode_brute_force_all_bf16_patterns(fmt):
    h = all_bf16_patterns()
    h = h[finite_mask(h)]
    v = bf16_bits_to_f64(h)
    want = brute_force_codes(fmt, v)
    got = oracle.fp8_encode_f32(fmt, v.astype(np.float32))
    bad = np.nonzero(want != got)[0]
    assert bad.size == 0, [(hex(h[i]), v[i], hex(want[i]), hex(got[i])) for i in bad[:8]]
    # the same through the fake-quant entry at scale 1 (bf16 input path)
    codes, deq = oracle.fake_quant_fp8(h, 1.0, 1.0, fmt)
    assert np.array_equal(codes, want)
    assert np.array_equal(deq.astype(np.float64), oracle.fp8_decode_table(fmt)[want])


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_encode_matches_library_cast_in_range(fmt):
    rng = np.random.default_rng(7)
    # fp32 values with full 23-bit mantissas, inside the finite range of the format
    mag = np.exp2(rng.uniform(EMIN[fmt] - MBITS[fmt] - 2, np.log2(FMAX[fmt]), 200000))
    y = (mag * rng.choice([-1.0, 1.0], mag.size)).astype(np.float32)
    y = y[np.abs(y) <= FMAX[fmt]]
    lib = torch.from_numpy(y).to(TORCH8[fmt]).view(torch.uint8).numpy()
    got = oracle.fp8_encode_f32(fmt, y)
    assert np.array_equal(lib, got)


@pytest.mark.parametrize("fmt", [oracle.E4M3, oracle.E5M2])
def test_encode_invariants(fmt):
    t = oracle.fp8_decode_table(fmt)
    h = all_bf16_patterns()
    h = h[finite_mask(h)]
    v = bf16_bits_to_f64(h).astype(np.float32)
    c = oracle.fp8_encode_f32(fmt, v)
    q = t[c]
    assert np.all(np.isfinite(q))
    # idempotent: Q(Q(x)) == Q(x); grid values have zero error
    assert np.array_equal(oracle.fp8_encode_f32(fmt, q.astype(np.float32)), c)
    grid = t[np.isfinite(t)].astype(np.float32)
    assert np.array_equal(t[oracle.fp8_encode_f32(fmt, grid)], grid.astype(np.float64))
    # odd symmetry
    assert np.array_equal(oracle.fp8_encode_f32(fmt, -v), c ^ 0x80)
    # monotone non-decreasing
    order = np.argsort(v.astype(np.float64), kind="stable")
    assert np.all(np.diff(q[order]) >= 0)
    # half-ulp bound inside the finite range
    inside = np.abs(v) <= FMAX[fmt]
    a = np.abs(v[inside].astype(np.float64))
    e = np.where(a > 0, np.floor(np.log2(np.where(a > 0, a, 1.0))), EMIN[fmt])
    e = np.maximum(e, EMIN[fmt])
    half_ulp = np.exp2(e - MBITS[fmt] - 1)
    assert np.all(np.abs(a - np.abs(q[inside])) <= half_ulp)
    # saturation outside
    assert np.all(np.abs(q[~inside]) == FMAX[fmt])
    # exact powers of two commute with Q away from the subnormal and saturation ends
    mid = (np.abs(v) >= 2.0 ** (EMIN[fmt] + 2)) & (np.abs(v) <= FMAX[fmt] / 8)
    for k in (-2, 1, 3):
        ck = oracle.fp8_encode_f32(fmt, (v[mid] * np.float32(2.0 ** k)))
        assert np.array_equal(t[ck], q[mid] * 2.0 ** k)


def test_bad_format_is_rejected():
    import ctypes as C
    tbl = np.empty(256)
    assert oracle.lib().orc_fp8_decode_table(C.c_int(9), tbl.ctypes.data_as(C.POINTER(C.c_double))) != 0
