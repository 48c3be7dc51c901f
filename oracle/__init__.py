"""ctypes face of the CPU oracle (oracle/ampsens_oracle.cpp).

TEST INFRASTRUCTURE: imported only by tests/, the smoke check and the benchmark's
cpu_baseline leg.  Argument marshalling only; every number comes from the C++ file.
bf16 tensors travel as numpy uint16 arrays.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

E4M3 = 0
E5M2 = 1

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.orc_fp8_max.restype = C.c_double
        L.orc_alpha.restype = C.c_double
        L.orc_layer_sensitivity.restype = C.c_double
        L.orc_fp8_max.argtypes = [C.c_int]
        L.orc_alpha.argtypes = [C.c_int]
        _lib = L
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def fp8_decode_table(fmt):
    t = np.empty(256, dtype=np.float64)
    rc = lib().orc_fp8_decode_table(C.c_int(fmt), _p(t, C.c_double))
    assert rc == 0
    return t


def fp8_max(fmt):
    return lib().orc_fp8_max(fmt)


def fp8_mantissa_bits(fmt):
    return lib().orc_fp8_mantissa_bits(C.c_int(fmt))


def alpha(mantissa_bits):
    return lib().orc_alpha(mantissa_bits)


def fp8_encode_f32(fmt, y):
    y = np.ascontiguousarray(y, dtype=np.float32)
    out = np.empty(y.size, dtype=np.uint8)
    rc = lib().orc_fp8_encode_f32(C.c_int(fmt), _p(y, C.c_float), C.c_int64(y.size),
                                  _p(out, C.c_uint8))
    assert rc == 0
    return out.reshape(y.shape)


def bf16_to_f32(x):
    x = _u16(x)
    out = np.empty(x.size, dtype=np.float32)
    lib().orc_bf16_to_f32(_p(x, C.c_uint16), C.c_int64(x.size), _p(out, C.c_float))
    return out.reshape(x.shape)


def absmax_scale(x, fmt, causal=None):
    """causal = (batch, rows, cols) or None.  Returns (amax, scale, inv, flags)."""
    x = _u16(x)
    am, sc, iv = C.c_float(), C.c_float(), C.c_float()
    fl = C.c_uint32()
    b, r, c = causal if causal else (0, 0, 0)
    rc = lib().orc_absmax_scale(_p(x, C.c_uint16), C.c_int64(x.size), C.c_int(1 if causal else 0),
                                C.c_int64(b), C.c_int64(r), C.c_int64(c), C.c_int(fmt),
                                C.byref(am), C.byref(sc), C.byref(iv), C.byref(fl))
    assert rc == 0
    return np.float32(am.value), np.float32(sc.value), np.float32(iv.value), fl.value


def scale_pow2(amax_bits, fmt):
    """(scale, inv) float32: the smallest power of two s with amax / s <= FMAX, and 1 / s."""
    sc, iv = C.c_float(), C.c_float()
    rc = lib().orc_scale_pow2(C.c_uint16(int(amax_bits)), int(fmt), C.byref(sc), C.byref(iv))
    assert rc == 0
    return np.float32(sc.value), np.float32(iv.value)


def fake_quant_fp8(x, scale, inv, fmt, want_dequant=True):
    x = _u16(x)
    codes = np.empty(x.size, dtype=np.uint8)
    deq = np.empty(x.size, dtype=np.float32) if want_dequant else None
    rc = lib().orc_fake_quant_fp8(_p(x, C.c_uint16), C.c_int64(x.size), C.c_float(scale),
                                  C.c_float(inv), C.c_int(fmt), _p(codes, C.c_uint8),
                                  _p(deq, C.c_float) if want_dequant else None)
    assert rc == 0
    return codes.reshape(x.shape), (deq.reshape(x.shape) if want_dequant else None)


def sens_operand(x, dx, R, n, scale, inv, fmt, x_shared=False, causal=None):
    """x: [R*stride] (or [stride] when x_shared), dx: [R*stride].  Returns (E[R], A[R])."""
    x, dx = _u16(x), _u16(dx)
    b, r, c = causal if causal else (0, 0, 0)
    stride = b * r * c if causal else n
    assert dx.size == R * stride
    assert x.size == (stride if x_shared else R * stride)
    E = np.empty(R, dtype=np.float64)
    A = np.empty(R, dtype=np.float64)
    rc = lib().orc_sens_operand(_p(x, C.c_uint16), _p(dx, C.c_uint16), C.c_int(R),
                                C.c_int64(0 if x_shared else stride), C.c_int64(stride),
                                C.c_int64(n), C.c_int(1 if causal else 0), C.c_int64(b),
                                C.c_int64(r), C.c_int64(c), C.c_float(scale), C.c_float(inv),
                                C.c_int(fmt), _p(E, C.c_double), _p(A, C.c_double))
    assert rc == 0
    return E, A


def absmax_scale_rows(x, n_rows, row_len, fmt, causal_rows=None):
    """Per-row (amax, scale, inv) float32 arrays [n_rows] and the flag word.  causal_rows: the
    operand is a stack of [causal_rows, row_len] matrices of which row i owns its first
    i + 1 + (row_len - causal_rows) entries."""
    x = _u16(x)
    assert x.size >= n_rows * row_len
    am = np.empty(n_rows, dtype=np.float32)
    sc = np.empty(n_rows, dtype=np.float32)
    iv = np.empty(n_rows, dtype=np.float32)
    fl = C.c_uint32()
    rc = lib().orc_absmax_scale_rows(_p(x, C.c_uint16), C.c_int64(n_rows), C.c_int64(row_len),
                                     0 if causal_rows is None else 1, C.c_int64(causal_rows or 0), int(fmt),
                                     _p(am, C.c_float), _p(sc, C.c_float), _p(iv, C.c_float), C.byref(fl))
    assert rc == 0
    return am, sc, iv, fl.value


def absmax_scale_blocks(x, n_rows, row_len, block, fmt):
    """(amax, scale, inv) float32 arrays [n_rows, row_len // block] of the 1 x block tiles, and the flag word."""
    x = _u16(x)
    assert x.size >= n_rows * row_len and row_len % block == 0
    shape = (n_rows, row_len // block)
    am = np.empty(shape, dtype=np.float32)
    sc = np.empty(shape, dtype=np.float32)
    iv = np.empty(shape, dtype=np.float32)
    fl = C.c_uint32()
    rc = lib().orc_absmax_scale_blocks(_p(x, C.c_uint16), C.c_int64(n_rows), C.c_int64(row_len), C.c_int64(block),
                                       int(fmt), _p(am, C.c_float), _p(sc, C.c_float), _p(iv, C.c_float), C.byref(fl))
    assert rc == 0
    return am, sc, iv, fl.value


def sens_operand_blocks(x, dx, n_rows, row_len, block, scale, inv, fmt):
    """(E, A) of one sample's [n_rows, row_len] block, tile (i, b) cast with scale[i, b], inv[i, b]."""
    x, dx = _u16(x), _u16(dx)
    scale = np.ascontiguousarray(scale, dtype=np.float32)
    inv = np.ascontiguousarray(inv, dtype=np.float32)
    assert x.size >= n_rows * row_len and dx.size >= n_rows * row_len and row_len % block == 0
    assert scale.size == n_rows * (row_len // block) and inv.size == scale.size
    E, A = C.c_double(), C.c_double()
    rc = lib().orc_sens_operand_blocks(_p(x, C.c_uint16), _p(dx, C.c_uint16), C.c_int64(n_rows), C.c_int64(row_len),
                                       C.c_int64(block), _p(scale, C.c_float), _p(inv, C.c_float), int(fmt),
                                       C.byref(E), C.byref(A))
    assert rc == 0
    return E.value, A.value


def sens_operand_rows(x, dx, n_rows, row_len, scale, inv, fmt, causal_rows=None):
    """(E, A) of one sample's [n_rows, row_len] block, row i cast with scale[i], inv[i]."""
    x, dx = _u16(x), _u16(dx)
    scale = np.ascontiguousarray(scale, dtype=np.float32)
    inv = np.ascontiguousarray(inv, dtype=np.float32)
    assert x.size >= n_rows * row_len and dx.size >= n_rows * row_len
    assert scale.size == n_rows and inv.size == n_rows
    E, A = C.c_double(), C.c_double()
    rc = lib().orc_sens_operand_rows(_p(x, C.c_uint16), _p(dx, C.c_uint16), C.c_int64(n_rows),
                                     C.c_int64(row_len), 0 if causal_rows is None else 1,
                                     C.c_int64(causal_rows or 0), _p(scale, C.c_float), _p(inv, C.c_float),
                                     int(fmt), C.byref(E), C.byref(A))
    assert rc == 0
    return E.value, A.value


def sens_linear(x, dx, w, dw, C_, K, R, row_off, x_scale, x_inv, w_scale, w_inv, fmt):
    """Returns out[R,4] = (E_X, A_X, E_W, A_W) per sample."""
    x, dx, w, dw = _u16(x), _u16(dx), _u16(w), _u16(dw)
    row_off = np.ascontiguousarray(row_off, dtype=np.int64)
    assert row_off.size == R + 1
    assert x.size == row_off[-1] * C_ == dx.size
    assert w.size == K * C_ and dw.size == R * K * C_
    out = np.empty((R, 4), dtype=np.float64)
    rc = lib().orc_sens_linear(_p(x, C.c_uint16), _p(dx, C.c_uint16), _p(w, C.c_uint16),
                               _p(dw, C.c_uint16), C.c_int64(C_), C.c_int64(K), C.c_int(R),
                               _p(row_off, C.c_int64), C.c_float(x_scale), C.c_float(x_inv),
                               C.c_float(w_scale), C.c_float(w_inv), C.c_int(fmt),
                               _p(out, C.c_double))
    assert rc == 0
    return out


def sens_bgemm(x0, dx0, lay0, x1, dx1, lay1, R, s0, i0, s1, i1, fmt):
    """lay = ('dense', n) or ('causal', batch, rows, cols).  Returns out[R,4]."""
    x0, dx0, x1, dx1 = _u16(x0), _u16(dx0), _u16(x1), _u16(dx1)

    def unpack(lay):
        if lay[0] == "dense":
            return (lay[1], 0, 0, 0, 0)
        return (0, 1, lay[1], lay[2], lay[3])

    n0, c0, b0, r0, k0 = unpack(lay0)
    n1, c1, b1, r1, k1 = unpack(lay1)
    out = np.empty((R, 4), dtype=np.float64)
    rc = lib().orc_sens_bgemm(_p(x0, C.c_uint16), _p(dx0, C.c_uint16), C.c_int64(n0), C.c_int(c0),
                              C.c_int64(b0), C.c_int64(r0), C.c_int64(k0), _p(x1, C.c_uint16),
                              _p(dx1, C.c_uint16), C.c_int64(n1), C.c_int(c1), C.c_int64(b1),
                              C.c_int64(r1), C.c_int64(k1), C.c_int(R), C.c_float(s0),
                              C.c_float(i0), C.c_float(s1), C.c_float(i1), C.c_int(fmt),
                              _p(out, C.c_double))
    assert rc == 0
    return out


def layer_sensitivity(A0, A1):
    A0 = np.ascontiguousarray(A0, dtype=np.float64)
    A1 = np.ascontiguousarray(A1, dtype=np.float64)
    return lib().orc_layer_sensitivity(_p(A0, C.c_double), _p(A1, C.c_double), C.c_int(A0.size))


def group_mse(s, alphas):
    s = np.ascontiguousarray(s, dtype=np.float64)
    alphas = np.ascontiguousarray(alphas, dtype=np.float64)
    d = np.empty(alphas.size ** s.size, dtype=np.float64)
    lib().orc_group_mse(_p(s, C.c_double), C.c_int(s.size), _p(alphas, C.c_double),
                        C.c_int(alphas.size), _p(d, C.c_double))
    return d


def _select(fn, n_choices, gain, mse, budget, extra=()):
    n_choices = np.ascontiguousarray(n_choices, dtype=np.int32)
    gain = np.ascontiguousarray(gain, dtype=np.float64)
    mse = np.ascontiguousarray(mse, dtype=np.float64)
    assert gain.size == mse.size == int(n_choices.sum())
    J = n_choices.size
    choice = np.zeros(J, dtype=np.int32)
    tg, td = C.c_double(), C.c_double()
    rc = fn(C.c_int(J), _p(n_choices, C.c_int32), _p(gain, C.c_double), _p(mse, C.c_double),
            C.c_double(budget), *extra, _p(choice, C.c_int32), C.byref(tg), C.byref(td))
    return rc, choice, tg.value, td.value


def select_exhaustive(n_choices, gain, mse, budget):
    return _select(lib().orc_select_exhaustive, n_choices, gain, mse, budget)


def select_pareto(n_choices, gain, mse, budget, max_states=5_000_000):
    return _select(lib().orc_select_pareto, n_choices, gain, mse, budget,
                   extra=(C.c_int64(max_states),))
