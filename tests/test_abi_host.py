"""Host-side checks of libampsens that need no GPU: the library loads and exports every symbol
the header declares; argument validation answers before any launch; the host replay of the
kernels' element walk visits every element of a unit exactly once and stays inside it; the
host epilogue and the selection solver agree with the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import paper_2505_13060_amd as amp
from conftest import host_hooks

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ampsens.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(amp_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert {"amp_absmax_scale", "amp_fake_quant_fp8", "amp_sens_linear", "amp_sens_bgemm",
            "amp_select_subgraphs"} <= set(names)
    L = amp.lib()
    for n in names:
        assert hasattr(L, n), n
    assert amp.amp_version() >= 100
    assert L.amp_status_string(amp.ERR_INFEASIBLE).decode().startswith("no configuration")


def test_product_library_exports_no_test_hooks():
    """Replay and schedule checks live in tests/host_hooks.cpp; the product ABI is the header, nothing more."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", amp._build.LIB], capture_output=True, text=True, check=True).stdout
    names = [line.split()[-1] for line in out.splitlines() if line.strip()]
    assert not [n for n in names if "debug" in n or n.startswith("hooks_")]
    exported = sorted(n for n in names if n.startswith("amp_"))
    assert exported == declared_symbols(), set(exported) ^ set(declared_symbols())


def test_budget_of_eq_ip():
    losses = np.array([0.5, -2.0, 3.0, 1.25])
    m = amp.amp_loss_second_moment(losses)
    assert m == pytest.approx((0.25 + 4.0 + 9.0 + 1.5625) / 4, rel=1e-15)
    assert amp.amp_mse_budget(0.01, m) == pytest.approx(1e-4 * m, rel=1e-15)
    assert amp.amp_mse_budget(0.0, m) == 0.0
    assert np.isnan(amp.amp_loss_second_moment(np.zeros(0)))


def test_struct_sizes_match_header():
    # natural C layout of the header's structs
    assert C.sizeof(amp.Layout) == 40
    assert C.sizeof(amp.Tensor) == 56
    assert C.sizeof(amp.LinearDesc) == 104
    assert C.sizeof(amp.BgemmDesc) == 152
    assert C.sizeof(amp.Plan) == 512


def test_argument_validation_without_a_gpu():
    L = amp.lib()
    n = C.c_size_t()
    fm = (C.c_int * 2)(0, 1)
    # bad format / format count
    assert L.amp_fake_quant_fp8(8, 16, 1.0, 1.0, 7, 8, None, None) == amp.ERR_BAD_FORMAT
    assert L.amp_absmax_scale(None, 0, fm, 3, None, None, None, None, None, 0, None) == amp.ERR_BAD_FORMAT
    assert L.amp_sens_linear(None, 0, (C.c_int * 1)(5), 1, None, None, 0, None) == amp.ERR_BAD_FORMAT
    # the power-of-two scale flag
    pw = (C.c_int * 2)(0 | amp.SCALE_POW2, 1 | amp.SCALE_POW2)
    assert L.amp_absmax_scale(None, 0, pw, 2, None, None, None, None, None, 0, None) == amp.OK
    assert L.amp_absmax_scale_rows(None, 0, pw, 2, None, None, None, None, None, 0, None) == amp.OK
    assert L.amp_sens_linear(None, 0, pw, 2, None, None, 0, None) == amp.OK     # the rule serves AMP_ROWS_COMPUTE operands
    assert L.amp_absmax_scale(None, 0, (C.c_int * 1)(2 | amp.SCALE_POW2), 1, None, None, None, None, None, 0, None) == amp.ERR_BAD_FORMAT
    # nothing to do is fine and launches nothing
    assert L.amp_fake_quant_fp8(None, 0, 1.0, 1.0, 0, None, None, None) == amp.OK
    assert L.amp_absmax_scale(None, 0, fm, 2, None, None, None, None, None, 0, None) == amp.OK
    assert L.amp_sens_linear(None, 0, fm, 2, None, None, 0, None) == amp.OK
    assert L.amp_sens_bgemm(None, 0, fm, 2, None, None, 0, None) == amp.OK
    # null / negative / misaligned
    assert L.amp_fake_quant_fp8(None, 16, 1.0, 1.0, 0, 8, None, None) == amp.ERR_INVALID_ARG
    assert L.amp_fake_quant_fp8(8, -1, 1.0, 1.0, 0, 8, None, None) == amp.ERR_INVALID_ARG
    assert L.amp_fake_quant_fp8(9, 16, 1.0, 1.0, 0, 8, None, None) == amp.ERR_INVALID_ARG
    assert L.amp_sens_linear(None, 1, fm, 2, None, None, 0, None) == amp.ERR_INVALID_ARG
    t = amp.Tensor(None, amp.dense(100), 1)
    assert L.amp_absmax_workspace_bytes(C.byref(t), 1, C.byref(n)) == amp.ERR_INVALID_ARG
    t = amp.Tensor(4096, amp.dense(-5), 1)
    assert L.amp_absmax_workspace_bytes(C.byref(t), 1, C.byref(n)) == amp.ERR_INVALID_ARG
    t = amp.Tensor(4096, amp.causal(1, 1 << 31, 8), 1)
    assert L.amp_absmax_workspace_bytes(C.byref(t), 1, C.byref(n)) == amp.ERR_TOO_LARGE
    # workspace: size query, then too small / misaligned / missing
    t = amp.Tensor(4096, amp.dense(1 << 20), 1)
    assert L.amp_absmax_workspace_bytes(C.byref(t), 1, C.byref(n)) == amp.OK and n.value >= 64 + 8 + 4
    args = (C.byref(t), 1, fm, 2, 256, 256, 256, 256)
    assert L.amp_absmax_scale(*args, 4096, n.value - 1, None) == amp.ERR_WORKSPACE_TOO_SMALL
    assert L.amp_absmax_scale(*args, 4100, n.value, None) == amp.ERR_INVALID_ARG
    assert L.amp_absmax_scale(*args, None, n.value, None) == amp.ERR_INVALID_ARG
    # linear descriptor consistency: offsets must start at 0 and not decrease
    off = np.array([0, 5, 3], dtype=np.int64)
    d = amp.linear_desc(None, None, None, None, 8, 8, 2, None, None, None, None, sample_row_offsets=off)
    d.x = d.dx = d.w = d.dw = 4096
    d.x_scale = d.x_inv = d.w_scale = d.w_inv = 4096
    assert L.amp_sens_linear_workspace_bytes(C.byref(d), 1, 2, C.byref(n)) == amp.ERR_INVALID_ARG
    off[:] = [0, 3, 5]
    assert L.amp_sens_linear_workspace_bytes(C.byref(d), 1, 2, C.byref(n)) == amp.OK
    # 4 units (X and W of 2 samples), one chunk each: uploaded table, resolved units, chunk map,
    # per-wave partials, each rounded up to 256 bytes
    assert n.value == 512 + 256 + 256 + 256


def test_block_call_is_validated_like_its_two_halves():
    """amp_sens_block: the workspace holds one table for all units; a bad descriptor on either side,
    a bad format or a short workspace is refused before any launch; nothing to do is not an error."""
    L = amp.lib()
    n, nl, nb = C.c_size_t(), C.c_size_t(), C.c_size_t()
    d = amp.linear_desc(None, None, None, None, 64, 32, 2, None, None, None, None, tokens=5)
    d.x = d.dx = d.w = d.dw = 4096
    d.x_scale = d.x_inv = d.w_scale = d.w_inv = 4096
    b = amp.bgemm_desc(None, None, amp.dense(4 * 64 * 16), None, None, amp.causal(4, 64, 64), 3,
                       None, None, None, None)
    b.x0 = b.dx0 = b.x1 = b.dx1 = 4096
    b.scale0 = b.inv0 = b.scale1 = b.inv1 = 4096
    assert L.amp_sens_block_workspace_bytes(C.byref(d), 1, C.byref(b), 1, 2, C.byref(n)) == amp.OK
    assert L.amp_sens_linear_workspace_bytes(C.byref(d), 1, 2, C.byref(nl)) == amp.OK
    assert L.amp_sens_bgemm_workspace_bytes(C.byref(b), 1, 2, C.byref(nb)) == amp.OK
    assert max(nl.value, nb.value) < n.value <= nl.value + nb.value
    assert L.amp_sens_block_workspace_bytes(C.byref(d), 1, None, 0, 2, C.byref(n)) == amp.OK and n.value == nl.value
    assert L.amp_sens_block_workspace_bytes(None, 0, C.byref(b), 1, 2, C.byref(n)) == amp.OK and n.value == nb.value
    assert L.amp_sens_block_workspace_bytes(None, 1, C.byref(b), 1, 2, C.byref(n)) == amp.ERR_INVALID_ARG
    assert L.amp_sens_block_workspace_bytes(C.byref(d), 1, C.byref(b), 1, 3, C.byref(n)) == amp.ERR_BAD_FORMAT
    fm = (C.c_int * 2)(amp.E4M3, amp.E5M2)
    bad = (C.c_int * 2)(amp.E4M3, 7)
    assert L.amp_sens_block(None, 0, None, 0, fm, 2, None, None, 0, None) == amp.OK
    assert L.amp_sens_block(C.byref(d), 1, C.byref(b), 1, bad, 2, 4096, 4096, 1 << 20, None) == amp.ERR_BAD_FORMAT
    assert L.amp_sens_block_workspace_bytes(C.byref(d), 1, C.byref(b), 1, 2, C.byref(n)) == amp.OK
    assert L.amp_sens_block(C.byref(d), 1, C.byref(b), 1, fm, 2, 4096, 4096, n.value - 1, None) == amp.ERR_WORKSPACE_TOO_SMALL
    assert L.amp_sens_block(C.byref(d), 1, C.byref(b), 1, fm, 2, None, 4096, n.value, None) == amp.ERR_INVALID_ARG
    b.R = -1
    assert L.amp_sens_block(C.byref(d), 1, C.byref(b), 1, fm, 2, 4096, 4096, n.value, None) == amp.ERR_INVALID_ARG
    b.R = 3
    d.scale_rows = 8                                           # a weight's scales are never computed by the pass
    assert L.amp_sens_block(C.byref(d), 1, C.byref(b), 1, fm, 2, 4096, 4096, n.value, None) == amp.ERR_INVALID_ARG


REPLAY_CASES = [
    # (layout, x offset in bytes from a 16-byte boundary, dx offset, batch_mul)
    (("dense", 1), 0, 0, 1), (("dense", 7), 0, 0, 1), (("dense", 8), 0, 0, 1),
    (("dense", 32768), 0, 0, 1), (("dense", 32769), 0, 0, 1), (("dense", 32767), 0, 0, 1),
    (("dense", 100000), 6, 6, 1), (("dense", 32768 * 3), 14, 14, 1), (("dense", 3), 10, 10, 1),
    (("dense", 40000), 2, 4, 1), (("dense", 123), 0, 8, 1), (("dense", 5000), 0, 0, 7), (("dense", 32768 * 2 + 8), 2, 2, 1),
    (("causal", 3, 64, 64), 0, 0, 1), (("causal", 2, 40, 40), 0, 0, 2), (("causal", 1, 37, 48), 0, 0, 1),
    (("causal", 2, 48, 24), 0, 0, 1), (("causal", 1, 33, 33), 0, 0, 1), (("causal", 2, 16, 72), 4, 4, 1),
    (("causal", 1, 100, 8), 0, 0, 1), (("causal", 1, 1, 1), 0, 0, 1), (("causal", 4, 8, 8), 0, 2, 1),
    (("causal", 1, 2048, 2048), 0, 0, 1), (("causal", 2, 520, 512), 0, 0, 1), (("causal", 1, 200, 1024), 0, 0, 3),
    (("causal", 3, 8, 16), 0, 0, 1), (("causal", 1, 31, 64), 0, 0, 1), (("causal", 2, 72, 8), 0, 0, 1),
    (("causal", 2, 512, 512), 0, 0, 1), (("causal", 1, 1024, 1024), 0, 0, 1), (("causal", 1, 4096, 4096), 0, 0, 1),
    (("causal", 2, 16, 16), 0, 0, 1), (("causal", 3, 24, 24), 0, 0, 1), (("causal", 1, 8, 8), 0, 0, 1),
    (("causal", 1, 1032, 1032), 0, 0, 1), (("causal", 1, 520, 1544), 0, 0, 1), (("causal", 1, 136, 136), 0, 0, 2),
    # odd and even band counts, bands that end inside, at the start and at the end of a 32-vector
    # group, rows that start empty, a ragged last band
    (("causal", 2, 256, 256), 0, 0, 1), (("causal", 1, 264, 264), 0, 0, 1), (("causal", 1, 248, 256), 0, 0, 1),
    (("causal", 1, 256, 264), 0, 0, 1), (("causal", 1, 300, 296), 0, 0, 1), (("causal", 1, 64, 512), 0, 0, 1),
    (("causal", 1, 250, 256), 0, 0, 1), (("causal", 1, 509, 768), 0, 0, 1), (("causal", 1, 776, 520), 0, 0, 1),
]


@pytest.mark.parametrize("lay,xo,dxo,mul", REPLAY_CASES)
def test_kernel_walk_covers_every_element_once(lay, xo, dxo, mul):
    L = host_hooks()
    if lay[0] == "dense":
        layout = amp.dense(lay[1])
        span = lay[1] * mul
        want = np.ones(span, dtype=np.int32)
    else:
        _, b, r, c = lay
        layout = amp.causal(b, r, c)
        span = b * r * c * mul
        i = np.arange(r)[:, None]
        j = np.arange(c)[None, :]
        want = np.broadcast_to((j <= i + (c - r)).astype(np.int32), (b * mul, r, c)).reshape(-1).copy()
    counts = np.zeros(span, dtype=np.int32)
    nch = C.c_uint64()
    bad = L.hooks_replay_unit(0x10000 + xo, 0x90000 + dxo, C.byref(layout), mul,
                                      counts.ctypes.data_as(C.c_void_p), span, C.byref(nch))
    assert bad == 0
    assert np.array_equal(counts, want)
    assert nch.value >= 1


ROW_REPLAY_CASES = [
    # (layout, row length, x offset, dx offset, batch_mul): dense [n / row_len, row_len] or causal rows
    (("dense", 4096 * 24), 4096, 0, 0, 1), (("dense", 11008 * 7), 11008, 0, 0, 1), (("dense", 128 * 700), 128, 0, 0, 1),
    (("dense", 8 * 5000), 8, 0, 0, 1), (("dense", 1408 * 50), 1408, 0, 0, 1), (("dense", 28672 * 3), 28672, 0, 0, 1),
    (("dense", 40 * 1000), 40, 0, 0, 2), (("dense", 32768 * 2), 32768, 0, 0, 1), (("dense", 65536 * 2), 65536, 0, 0, 1),
    (("dense", 256 * 400), 256, 0, 0, 1), (("dense", 64 * 3000), 64, 0, 0, 1), (("dense", 16 * 9000), 16, 0, 0, 1),
    (("dense", 520 * 130), 520, 0, 0, 1), (("dense", 1000 * 70), 1000, 0, 0, 1), (("dense", 48 * 1500), 48, 0, 0, 1),
    (("dense", 100 * 333), 100, 0, 0, 1),                     # row length not a multiple of 8: element path
    (("dense", 128 * 300), 128, 6, 6, 1),                     # misaligned buffer: element path
    (("dense", 4096 * 9), 4096, 0, 8, 1),                     # x and xdot misaligned against each other
    (("causal", 3, 64, 64), 64, 0, 0, 1), (("causal", 1, 37, 48), 48, 0, 0, 2), (("causal", 2, 520, 512), 512, 0, 0, 1),
    (("causal", 2, 16, 72), 72, 4, 4, 1), (("causal", 1, 200, 1024), 1024, 0, 0, 1),
]


@pytest.mark.parametrize("lay,row_len,xo,dxo,mul", ROW_REPLAY_CASES)
def test_kernel_walk_tracks_the_row_of_every_vector(lay, row_len, xo, dxo, mul):
    """Units with one scale per row: the replay of the kernels' index code also follows the row of
    every vector the way the device context does (one division per chunk, then additions; or the
    row named by the causal walker) and compares it with element index / row length."""
    L = host_hooks()
    if lay[0] == "dense":
        layout = amp.dense(lay[1])
        span = lay[1] * mul
        want = np.ones(span, dtype=np.int32)
    else:
        _, b, r, c = lay
        layout = amp.causal(b, r, c)
        span = b * r * c * mul
        i = np.arange(r)[:, None]
        j = np.arange(c)[None, :]
        want = np.broadcast_to((j <= i + (c - r)).astype(np.int32), (b * mul, r, c)).reshape(-1).copy()
    counts = np.zeros(span, dtype=np.int32)
    nch = C.c_uint64()
    bad = L.hooks_replay_unit_rows(0x10000 + xo, 0x90000 + dxo, C.byref(layout), mul, row_len,
                                           counts.ctypes.data_as(C.c_void_p), span, C.byref(nch))
    assert bad == 0
    assert np.array_equal(counts, want)


def test_row_scale_descriptors_are_validated():
    L = amp.lib()
    n = C.c_size_t()
    rows = C.c_int64()
    d = amp.linear_desc(None, None, None, None, 64, 32, 2, None, None, None, None, tokens=5, scale_rows=3)
    d.x = d.dx = d.w = d.dw = 4096
    d.x_scale = d.x_inv = d.w_scale = d.w_inv = 4096
    assert L.amp_sens_linear_workspace_bytes(C.byref(d), 1, 2, C.byref(n)) == amp.OK
    d.scale_rows = 8                                           # a weight's scales are never computed by the pass
    assert L.amp_sens_linear_workspace_bytes(C.byref(d), 1, 2, C.byref(n)) == amp.ERR_INVALID_ARG
    # scale blocks inside the rows: the block must divide C and some operand must have row scales
    for flags, want in ((3 | amp.rows_block(16), amp.OK), (1 | amp.rows_block(64), amp.OK), (2 | amp.rows_block(32), amp.OK),
                        (4 | amp.rows_block(8), amp.OK), (3 | amp.rows_block(48), amp.ERR_INVALID_ARG),
                        (amp.rows_block(16), amp.ERR_INVALID_ARG), (3 | amp.rows_block(128), amp.ERR_INVALID_ARG)):
        d.scale_rows = flags
        assert L.amp_sens_linear_workspace_bytes(C.byref(d), 1, 2, C.byref(n)) == want, hex(flags)
    # a dense BGEMM operand with one scale per row must say its row length, and it must divide the block
    b = amp.bgemm_desc(None, None, amp.dense(4 * 64 * 16), None, None, amp.dense(4 * 64 * 16, 16), 2,
                       None, None, None, None, scale_rows=amp.ROWS_OPERAND1)
    b.x0 = b.dx0 = b.x1 = b.dx1 = 4096
    b.scale0 = b.inv0 = b.scale1 = b.inv1 = 4096
    assert L.amp_sens_bgemm_workspace_bytes(C.byref(b), 1, 2, C.byref(n)) == amp.OK
    b.scale_rows = amp.ROWS_OPERAND0
    assert L.amp_sens_bgemm_workspace_bytes(C.byref(b), 1, 2, C.byref(n)) == amp.ERR_INVALID_ARG
    b.layout0 = amp.dense(4 * 64 * 16, 48)                     # 4096 % 48 != 0
    assert L.amp_sens_bgemm_workspace_bytes(C.byref(b), 1, 2, C.byref(n)) == amp.ERR_INVALID_ARG
    # rows of an absmax call
    t = amp.Tensor(4096, amp.dense(1000 * 128, 128), 3)
    assert L.amp_absmax_rows_workspace_bytes(C.byref(t), 1, C.byref(n), C.byref(rows)) == amp.OK
    assert rows.value == 3000 and n.value == 256
    t = amp.Tensor(4096, amp.causal(2, 40, 64), 3)
    assert L.amp_absmax_rows_workspace_bytes(C.byref(t), 1, C.byref(n), C.byref(rows)) == amp.OK
    assert rows.value == 240
    t = amp.Tensor(4096, amp.dense(1000), 1)                   # no row length
    assert L.amp_absmax_rows_workspace_bytes(C.byref(t), 1, C.byref(n), C.byref(rows)) == amp.ERR_INVALID_ARG
    fm = (C.c_int * 2)(0, 1)
    t = amp.Tensor(4096, amp.dense(1024, 128), 1)
    assert L.amp_absmax_scale_rows(C.byref(t), 1, fm, 2, 256, 256, 256, 256, 4096, 0, None) == amp.ERR_WORKSPACE_TOO_SMALL
    assert L.amp_absmax_scale_rows(C.byref(t), 1, fm, 2, 256, 256, 256, None, 4096, 256, None) == amp.ERR_INVALID_ARG
    assert L.amp_absmax_scale_rows(None, 0, fm, 2, None, None, None, None, None, 0, None) == amp.OK


@pytest.mark.parametrize("shapes", [
    [(4, 256, 1024, 1024)],                                   # config 0
    [(16, 2048, 4096, 4096), (16, 2048, 4096, 11008)],        # two linears of the 7B block
    [(3, 5, 8, 9), (1, 7, 64, 64), (5, 1, 4099, 33)],         # odd sizes: members differ in alignment
    [(32, 100, 512, 176)] * 6,                                # several small experts
])
def test_schedule_is_a_permutation_of_the_chunks(shapes):
    """Weight units of one op (same W, one gradient per sample) are interleaved in the schedule;
    whatever the shapes, every chunk must get exactly one position."""
    L = host_hooks()
    descs = []
    base = 0x100000
    for (R, tokens, Cd, K) in shapes:
        d = amp.LinearDesc()
        d.x = d.dx = d.w = base
        d.dw = base + 2                                        # 2 bytes off: alignment varies with r
        d.C, d.K, d.tokens, d.R = Cd, K, tokens, R
        d.x_scale = d.x_inv = d.w_scale = d.w_inv = base
        descs.append(d)
    arr = (amp.LinearDesc * len(descs))(*descs)
    n, inter = C.c_uint64(), C.c_uint64()
    for block, use_w in ((0, 1), (0, 0), (1, 1), (3, 0), (5, 1)):
        assert L.hooks_check_linear_schedule(arr, len(descs), 2, block, use_w, C.byref(n), C.byref(inter)) == 0
    assert n.value >= len(descs)
    if shapes[0][0] > 1 and shapes[0][2] * shapes[0][3] % 8 == 0:
        assert inter.value > 0


@pytest.mark.parametrize("shapes,ragged,max_records", [
    ([(16, 2048, 4096, 4096), (16, 2048, 4096, 11008), (16, 2048, 11008, 4096)], False, 6),   # x and w of each op: a run
    ([(4, 256, 1024, 1024)], False, 2),
    ([(32, 100, 512, 176)] * 6, True, None),                   # ragged samples: the x units do not repeat
    ([(3, 5, 8, 9), (1, 7, 64, 64), (5, 1, 4099, 33), (2, 9, 16, 16)], False, None),
])
def test_table_travels_as_runs_and_expands_to_the_same_bytes(shapes, ragged, max_records):
    """The unit table of a call, cut into runs of units whose fields advance by fixed steps plus
    literal units, expands to the table byte for byte; the samples of a uniform op collapse into one
    run per operand."""
    L = host_hooks()
    L.hooks_table_records.restype = C.c_int64
    descs, keep = [], []
    base = 0x100000
    rng = np.random.default_rng(11)
    for (R, tokens, Cd, K) in shapes:
        d = amp.LinearDesc()
        d.x = d.dx = d.w = base
        d.dw = base + 64
        d.C, d.K, d.tokens, d.R = Cd, K, tokens, R
        if ragged:
            offs = np.concatenate([[0], np.cumsum(rng.integers(1, tokens + 1, R))]).astype(np.int64)
            keep.append(offs)
            d.tokens = 0
            d.sample_row_offsets = offs.ctypes.data_as(C.POINTER(C.c_int64))
        d.x_scale = d.x_inv = d.w_scale = d.w_inv = base
        descs.append(d)
        base += 0x10000000
    arr = (amp.LinearDesc * len(descs))(*descs)
    runs, lits, raw, units = C.c_uint64(), C.c_uint64(), C.c_uint64(), C.c_uint64()
    bad = L.hooks_table_records(arr, len(descs), 2, C.byref(runs), C.byref(lits), C.byref(raw), C.byref(units))
    assert bad == 0
    assert units.value == 2 * sum(s_[0] for s_ in shapes)
    if max_records is not None:
        assert lits.value == 0 and runs.value <= max_records
    if ragged:
        assert lits.value > 0 and runs.value >= len(shapes)    # the weights' units still form runs


def test_epilogue_matches_oracle():
    rng = np.random.default_rng(4)
    R, nf = 5, 2
    sums = rng.uniform(0.1, 2.0, (R, nf, 4)).astype(np.float32)
    sums[:, 1, 1] = sums[:, 0, 1]
    sums[:, 1, 3] = sums[:, 0, 3]
    s, d_model, d_meas = amp.amp_layer_loss_mse(sums, [amp.E4M3, amp.E5M2])
    want_s = oracle.layer_sensitivity(sums[:, 0, 1].astype(np.float64), sums[:, 0, 3].astype(np.float64))
    assert s == pytest.approx(want_s, rel=1e-14)
    assert d_model[0] == pytest.approx(want_s * oracle.alpha(3), rel=1e-14)
    assert d_model[1] == pytest.approx(want_s * oracle.alpha(2), rel=1e-14)
    for f in range(nf):
        assert d_meas[f] == pytest.approx(float(np.mean(sums[:, f, 0].astype(np.float64) + sums[:, f, 2])), rel=1e-14)
    assert amp.amp_alpha(3) == oracle.alpha(3) == 1.0 / 768.0
    assert amp.amp_alpha(2) == oracle.alpha(2) == 1.0 / 192.0
    # group tables: d from the oracle's definition (same column order); gains add the same way
    s_layers = rng.uniform(0.5, 3.0, 4)
    alphas = np.array([0.0, oracle.alpha(3), oracle.alpha(2)])
    layer_mse = s_layers[:, None] * alphas[None, :]
    layer_gain = rng.uniform(0, 5, (4, 3))
    layer_gain[:, 0] = 0
    d, c = amp.amp_group_tables(layer_mse, layer_gain)
    assert np.allclose(d, oracle.group_mse(s_layers, alphas), rtol=1e-14, atol=0)
    for p in (0, 1, 17, 80):
        digits = [(p // 3 ** l) % 3 for l in range(4)]
        assert c[p] == pytest.approx(sum(layer_gain[l, digits[l]] for l in range(4)), rel=1e-14)


def offsets(n_choices):
    return np.concatenate([[0], np.cumsum(n_choices)])[:-1]


def check_against(solver_result, n_choices, gain, mse, budget, want_gain):
    choice, tg, td = solver_result
    off = offsets(n_choices)
    assert np.all((choice >= 0) & (choice < n_choices))
    assert gain[off + choice].sum() == pytest.approx(tg, rel=1e-12, abs=1e-12)
    assert mse[off + choice].sum() == pytest.approx(td, rel=1e-12, abs=1e-12)
    assert td <= budget * (1 + 1e-12) + 1e-300
    assert tg == pytest.approx(want_gain, rel=1e-11, abs=1e-12)


@pytest.mark.parametrize("seed", range(60))
def test_select_matches_oracle_enumeration(seed):
    rng = np.random.default_rng(seed)
    J = int(rng.integers(1, 7))
    n_choices = rng.integers(1, 6, J).astype(np.int32)
    gain = rng.uniform(-1, 10, n_choices.sum())
    mse = rng.uniform(0, 1, n_choices.sum())
    if seed % 2 == 0:
        gain[offsets(n_choices)] = 0.0
        mse[offsets(n_choices)] = 0.0
    budget = float(rng.uniform(0, mse.sum() * 0.5))
    rc, _, want_g, want_d = oracle.select_exhaustive(n_choices, gain, mse, budget)
    if rc != 0:
        with pytest.raises(amp.AmpError) as ei:
            amp.amp_select_subgraphs(n_choices, gain, mse, budget)
        assert ei.value.status == amp.ERR_INFEASIBLE
        return
    check_against(amp.amp_select_subgraphs(n_choices, gain, mse, budget), n_choices, gain, mse, budget, want_g)


def llama_like_instance(rng, blocks, budget_frac):
    """Groups of one decoder block as in the paper's Llama-3 partition (attention sub-graph with
    five quantisable ops, o_proj, {gate, up}, down; Appendix B figure), F = 3 formats."""
    alphas = np.array([0.0, 1.0 / 768.0, 1.0 / 192.0])
    n_choices, gains, mses = [], [], []
    for _ in range(blocks):
        for n_layers in (5, 1, 2, 1):
            s = np.exp(rng.normal(0, 1.5, n_layers))
            macs = np.exp(rng.normal(0, 0.7, n_layers))
            d = oracle.group_mse(s, alphas)
            layer_gain = np.stack([np.zeros(n_layers), 0.5 * macs, 0.5 * macs * (1 + 0.01 * rng.random(n_layers))], axis=1)
            _, c = amp.amp_group_tables(s[:, None] * alphas[None, :], layer_gain)
            n_choices.append(d.size)
            gains.append(c)
            mses.append(d)
    mse = np.concatenate(mses)
    budget = budget_frac * sum(m.max() for m in mses)
    return np.array(n_choices, dtype=np.int32), np.concatenate(gains), mse, float(budget)


@pytest.mark.parametrize("blocks,frac", [(2, 0.05), (4, 0.2), (8, 1e-3), (8, 0.3), (32, 1e-3), (32, 0.05)])
def test_select_matches_oracle_pareto_on_block_structured_instances(blocks, frac):
    rng = np.random.default_rng(blocks * 7 + int(frac * 1000))
    n_choices, gain, mse, budget = llama_like_instance(rng, blocks, frac)
    rc, _, want_g, _ = oracle.select_pareto(n_choices, gain, mse, budget, max_states=20_000_000)
    assert rc == 0
    check_against(amp.amp_select_subgraphs(n_choices, gain, mse, budget), n_choices, gain, mse, budget, want_g)


def lp_bound(n_choices, gain, mse, budget):
    """Upper bound of eq. (ip): its LP relaxation, by sorting the edges of every group's upper convex
    hull by slope (plain numpy, independent of the library)."""
    off = offsets(n_choices)
    base_d = base_g = 0.0
    edges = []
    for o, k in zip(off, n_choices):
        pts = sorted(zip(mse[o:o + k], gain[o:o + k]))
        keep = []
        best = -np.inf
        for d, g in pts:                                       # non-dominated, by increasing mse
            if g > best:
                keep.append((d, g))
                best = g
        hull = []
        for p in keep:
            while len(hull) >= 2 and (hull[-1][1] - hull[-2][1]) * (p[0] - hull[-2][0]) <= \
                    (p[1] - hull[-2][1]) * (hull[-1][0] - hull[-2][0]):
                hull.pop()
            hull.append(p)
        base_d += hull[0][0]
        base_g += hull[0][1]
        edges += [(b[0] - a[0], b[1] - a[1]) for a, b in zip(hull, hull[1:])]
    edges.sort(key=lambda e: -e[1] / e[0])
    room, g = budget - base_d, base_g
    greedy = base_g
    for dd, dg in edges:
        if dd <= room:
            room -= dd
            g += dg
            greedy = g
        else:
            g += dg * room / dd
            break
    return g, greedy


@pytest.mark.parametrize("blocks,sizes,frac", [(80, (5, 1, 2, 1), 0.1), (80, (1,) * 9, 0.02), (16, (1,) * 88, 0.1),
                                               (16, (1,) * 88, 0.5)])
def test_select_on_model_sized_instances_is_fast_and_within_the_lp_bound(blocks, sizes, frac):
    """70B-sized partitions and the 1408 single-layer groups of the ragged configuration: the optimum lies
    between the greedy walk along the hulls and the LP bound, which differ by one hull edge."""
    import time
    rng = np.random.default_rng(blocks + len(sizes))
    n_choices, gains, mses = [], [], []
    for _ in range(blocks):
        depth = np.exp(rng.normal(0, 0.7))
        for L in sizes:
            lm = np.zeros((L, 3))
            lg = np.zeros((L, 3))
            lm[:, 1] = rng.uniform(0.5, 2, L) * depth / 768
            lm[:, 2] = lm[:, 1] * 4 * rng.uniform(0.8, 1.2, L)
            lg[:, 1:] = rng.uniform(1, 10, L)[:, None]
            d, c = amp.amp_group_tables(lm, lg)
            n_choices.append(d.size)
            mses.append(d)
            gains.append(c)
    n_choices = np.array(n_choices, dtype=np.int32)
    gain, mse = np.concatenate(gains), np.concatenate(mses)
    budget = frac * sum(m.max() for m in mses)
    t0 = time.perf_counter()
    choice, tg, td = amp.amp_select_subgraphs(n_choices, gain, mse, budget)
    dt = time.perf_counter() - t0
    off = offsets(n_choices)
    assert td <= budget and mse[off + choice].sum() == pytest.approx(td, rel=1e-12)
    assert gain[off + choice].sum() == pytest.approx(tg, rel=1e-12)
    ub, greedy = lp_bound(n_choices, gain, mse, budget)
    assert greedy * (1 - 1e-12) <= tg <= ub * (1 + 1e-12)
    assert ub - tg <= 10.0 + 1e-9                              # one hull edge gains at most 10 here
    assert dt < 2.0


def test_select_invariances_and_errors():
    rng = np.random.default_rng(77)
    n_choices, gain, mse, budget = llama_like_instance(rng, 3, 0.1)
    choice, tg, td = amp.amp_select_subgraphs(n_choices, gain, mse, budget)
    # affine change of the gain (a > 0, one bias per group) keeps the arg max (Sec. 2.3.2)
    b = np.repeat(rng.uniform(-3, 3, n_choices.size), n_choices)
    choice2, tg2, td2 = amp.amp_select_subgraphs(n_choices, 2.5 * gain + b, mse, budget)
    assert gain[offsets(n_choices) + choice2].sum() == pytest.approx(tg, rel=1e-10)
    # tau = 0 -> all high precision; unlimited budget -> each group's best gain (Sec. 3.2)
    choice0, tg0, td0 = amp.amp_select_subgraphs(n_choices, gain, mse, 0.0)
    assert np.all(choice0 == 0) and tg0 == 0.0 and td0 == 0.0
    choice_inf, tgi, _ = amp.amp_select_subgraphs(n_choices, gain, mse, float(mse.sum()))
    off = np.concatenate([[0], np.cumsum(n_choices)])
    assert tgi == pytest.approx(sum(gain[off[j]:off[j + 1]].max() for j in range(n_choices.size)), rel=1e-12)
    # monotone in the budget
    prev = -1.0
    for frac in (0.0, 0.01, 0.05, 0.2, 0.5, 1.0):
        _, g, _ = amp.amp_select_subgraphs(n_choices, gain, mse, frac * budget * 10)
        assert g >= prev - 1e-12
        prev = g
    L = amp.lib()
    assert L.amp_select_subgraphs(1, None, None, None, C.c_double(1.0), None, None, None) == amp.ERR_INVALID_ARG
    bad = mse.copy()
    bad[3] = -1.0
    with pytest.raises(amp.AmpError):
        amp.amp_select_subgraphs(n_choices, gain, bad, budget)
    with pytest.raises(amp.AmpError) as ei:
        amp.amp_select_subgraphs(np.array([1], dtype=np.int32), np.array([1.0]), np.array([2.0]), 1.0)
    assert ei.value.status == amp.ERR_INFEASIBLE
