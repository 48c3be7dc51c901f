"""Python face of libampsens (include/ampsens.h): argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch appears here only as the
owner of device memory and streams.  There is no CPU fallback: if the shared library is
missing or fails to load, importing the binding's functions raises.
"""
import ctypes as C
import os

import numpy as np
import torch

from . import build as _build

E4M3 = 0
E5M2 = 1
MAX_FORMATS = 2
SCALE_POW2 = 0x100         # or-ed into a format for the absmax calls: power-of-two scales
ROWS_OPERAND0 = 1          # one scale per row of X (linear) / X0 (BGEMM)
ROWS_OPERAND1 = 2          # one scale per row of W (linear) / X1 (BGEMM)
ROWS_COMPUTE0 = 4          # operand 0: one scale per row, computed by the sensitivity pass itself (single read)
ROWS_COMPUTE1 = 8          # operand 1 of a BGEMM, likewise
ROWS_COMPUTE_MAX_ROW_LEN = 24576
PLAN_STREAM_WEIGHTS = 1    # amp_sens_block_setup flag: read W with every sample's gradient


def plan_interleave(n):
    """amp_sens_block_setup flag: chunks of one reader of a shared W next to each other in the schedule."""
    return (int(n) & 0xFF) << 8

OK, ERR_INVALID_ARG, ERR_BAD_FORMAT, ERR_WORKSPACE_TOO_SMALL, ERR_NONFINITE_INPUT, ERR_DEVICE, \
    ERR_INFEASIBLE, ERR_TOO_LARGE = range(8)


class AmpError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().amp_status_string(status).decode()
        if status == ERR_DEVICE:
            msg += " (hipError_t %d)" % lib().amp_last_device_error()
        super().__init__("%s: %s" % (where, msg))


class Plan(C.Structure):
    """amp_plan_t: what a run needs, filled by the *_setup calls; keeps the tensors it points into alive."""
    _fields_ = [("opaque", C.c_uint64 * 64)]


class Layout(C.Structure):
    _fields_ = [("n_elems", C.c_int64), ("batch", C.c_int64), ("rows", C.c_int64),
                ("cols", C.c_int64), ("causal", C.c_int32), ("reserved", C.c_int32)]


class Tensor(C.Structure):
    _fields_ = [("data", C.c_void_p), ("layout", Layout), ("n_samples", C.c_int64)]


class LinearDesc(C.Structure):
    _fields_ = [("x", C.c_void_p), ("dx", C.c_void_p), ("w", C.c_void_p), ("dw", C.c_void_p),
                ("C", C.c_int64), ("K", C.c_int64), ("tokens", C.c_int64),
                ("sample_row_offsets", C.POINTER(C.c_int64)), ("R", C.c_int32),
                ("scale_rows", C.c_int32), ("x_scale", C.c_void_p), ("x_inv", C.c_void_p),
                ("w_scale", C.c_void_p), ("w_inv", C.c_void_p)]


class BgemmDesc(C.Structure):
    _fields_ = [("x0", C.c_void_p), ("dx0", C.c_void_p), ("x1", C.c_void_p), ("dx1", C.c_void_p),
                ("layout0", Layout), ("layout1", Layout), ("R", C.c_int32), ("scale_rows", C.c_int32),
                ("scale0", C.c_void_p), ("inv0", C.c_void_p), ("scale1", C.c_void_p),
                ("inv1", C.c_void_p)]


_lib = None


def lib():
    """The loaded C-ABI library; built in-tree by build.py if no binary is there."""
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        L = C.CDLL(path)
        L.amp_status_string.restype = C.c_char_p
        L.amp_status_string.argtypes = [C.c_int]
        L.amp_alpha.restype = C.c_double
        L.amp_alpha.argtypes = [C.c_int]
        L.amp_fake_quant_fp8.argtypes = [C.c_void_p, C.c_int64, C.c_float, C.c_float, C.c_int,
                                         C.c_void_p, C.c_void_p, C.c_void_p]
        L.amp_absmax_scale.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                       C.c_void_p]
        L.amp_absmax_workspace_bytes.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_size_t)]
        L.amp_absmax_scale_rows.argtypes = L.amp_absmax_scale.argtypes
        L.amp_absmax_rows_workspace_bytes.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_size_t),
                                                      C.POINTER(C.c_int64)]
        for name in ("amp_sens_linear", "amp_sens_bgemm"):
            getattr(L, name).argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p,
                                         C.c_void_p, C.c_size_t, C.c_void_p]
            getattr(L, name + "_workspace_bytes").argtypes = [C.c_void_p, C.c_int, C.c_int,
                                                              C.POINTER(C.c_size_t)]
        L.amp_sens_block.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p,
                                     C.c_void_p, C.c_size_t, C.c_void_p]
        L.amp_sens_block_workspace_bytes.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                                     C.POINTER(C.c_size_t)]
        setup_tail = [C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(Plan)]
        for name in ("amp_absmax_scale_setup", "amp_absmax_scale_rows_setup"):
            getattr(L, name).argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_void_p] + setup_tail
        L.amp_sens_block_setup.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_int,
                                           C.c_void_p, C.c_void_p, C.c_size_t, C.c_uint32, C.c_void_p,
                                           C.POINTER(Plan)]
        L.amp_sens_block_static.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_int,
                                            C.c_void_p, C.c_void_p]
        L.amp_plan_limit_grid.argtypes = [C.POINTER(Plan), C.c_int]
        L.amp_run.argtypes = [C.POINTER(Plan), C.c_void_p]
        _lib = L
    return _lib


def _check(status, where):
    if status != OK:
        raise AmpError(status, where)


def _fmts(fmts):
    arr = (C.c_int * len(fmts))(*[int(f) for f in fmts])
    return arr, len(fmts)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _ptr(t):
    return None if t is None else t.data_ptr()


def rows_block(n):
    """AMP_ROWS_BLOCK(n): or into scale_rows to cut the rows of the row-scaled operands into 1 x n scale blocks."""
    n = int(n)
    assert 0 < n < (1 << 23)
    return n << 8


def dense(n_elems, cols=0):
    """cols: row length, needed only where the operand has one scale per row."""
    return Layout(int(n_elems), 0, 0, int(cols), 0, 0)


def causal(batch, rows, cols):
    return Layout(0, int(batch), int(rows), int(cols), 1, 0)


def tensor(data, layout, n_samples=1):
    """amp_tensor_t for amp_absmax_scale.  `data` is a bf16 (or int16/uint16 view) device tensor."""
    return Tensor(_ptr(data), layout, int(n_samples))


def linear_desc(x, dx, w, dw, C_, K, R, x_scale, x_inv, w_scale, w_inv, tokens=0,
                sample_row_offsets=None, scale_rows=0):
    d = LinearDesc()
    d.scale_rows = int(scale_rows)
    d.x, d.dx, d.w, d.dw = _ptr(x), _ptr(dx), _ptr(w), _ptr(dw)
    d.C, d.K, d.tokens, d.R = int(C_), int(K), int(tokens), int(R)
    if sample_row_offsets is not None:
        off = np.ascontiguousarray(sample_row_offsets, dtype=np.int64)
        d._keep = off                                   # keep the host array alive
        d.sample_row_offsets = off.ctypes.data_as(C.POINTER(C.c_int64))
    d.x_scale, d.x_inv, d.w_scale, d.w_inv = _ptr(x_scale), _ptr(x_inv), _ptr(w_scale), _ptr(w_inv)
    return d


def bgemm_desc(x0, dx0, layout0, x1, dx1, layout1, R, scale0, inv0, scale1, inv1, scale_rows=0):
    d = BgemmDesc()
    d.scale_rows = int(scale_rows)
    d.x0, d.dx0, d.x1, d.dx1 = _ptr(x0), _ptr(dx0), _ptr(x1), _ptr(dx1)
    d.layout0, d.layout1, d.R = layout0, layout1, int(R)
    d.scale0, d.inv0, d.scale1, d.inv1 = _ptr(scale0), _ptr(inv0), _ptr(scale1), _ptr(inv1)
    return d


def _array(cls, items):
    arr = (cls * max(len(items), 1))()
    for i, it in enumerate(items):
        arr[i] = it
    arr._keep = list(items)
    return arr


def amp_absmax_workspace_bytes(tensors):
    n = C.c_size_t()
    _check(lib().amp_absmax_workspace_bytes(_array(Tensor, tensors), len(tensors), C.byref(n)),
           "amp_absmax_workspace_bytes")
    return n.value


def amp_absmax_scale(tensors, fmts, d_amax, d_scale, d_inv, d_flags, workspace, stream=None):
    """tensors: list of Tensor.  d_amax [n] f32, d_scale / d_inv [n, n_fmts] f32, d_flags [n] i32,
    workspace: uint8 device tensor."""
    f, nf = _fmts(fmts)
    _check(lib().amp_absmax_scale(_array(Tensor, tensors), len(tensors), f, nf, _ptr(d_amax),
                                  _ptr(d_scale), _ptr(d_inv), _ptr(d_flags), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream(stream)),
           "amp_absmax_scale")


def amp_absmax_rows_workspace_bytes(tensors):
    """Returns (workspace bytes, total number of rows)."""
    n, rows = C.c_size_t(), C.c_int64()
    _check(lib().amp_absmax_rows_workspace_bytes(_array(Tensor, tensors), len(tensors), C.byref(n),
                                                 C.byref(rows)), "amp_absmax_rows_workspace_bytes")
    return n.value, rows.value


def amp_absmax_scale_rows(tensors, fmts, d_amax, d_scale, d_inv, d_flags, workspace, stream=None):
    """One scale per row: d_amax [rows] f32, d_scale / d_inv [rows, n_fmts] f32 over the rows of all
    tensors in order, d_flags [n_tensors] i32."""
    f, nf = _fmts(fmts)
    _check(lib().amp_absmax_scale_rows(_array(Tensor, tensors), len(tensors), f, nf, _ptr(d_amax),
                                       _ptr(d_scale), _ptr(d_inv), _ptr(d_flags), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream(stream)),
           "amp_absmax_scale_rows")


def amp_fake_quant_fp8(d_x, n, scale, inv_scale, fmt, d_codes, d_dequant=None, stream=None):
    _check(lib().amp_fake_quant_fp8(_ptr(d_x), int(n), float(scale), float(inv_scale), int(fmt),
                                    _ptr(d_codes), _ptr(d_dequant), _stream(stream)),
           "amp_fake_quant_fp8")


def amp_sens_linear_workspace_bytes(ops, n_fmts):
    n = C.c_size_t()
    _check(lib().amp_sens_linear_workspace_bytes(_array(LinearDesc, ops), len(ops), int(n_fmts),
                                                 C.byref(n)), "amp_sens_linear_workspace_bytes")
    return n.value


def amp_sens_linear(ops, fmts, d_out, workspace, stream=None):
    f, nf = _fmts(fmts)
    _check(lib().amp_sens_linear(_array(LinearDesc, ops), len(ops), f, nf, _ptr(d_out),
                                 _ptr(workspace), workspace.numel() * workspace.element_size(),
                                 _stream(stream)), "amp_sens_linear")


def amp_sens_bgemm_workspace_bytes(ops, n_fmts):
    n = C.c_size_t()
    _check(lib().amp_sens_bgemm_workspace_bytes(_array(BgemmDesc, ops), len(ops), int(n_fmts),
                                                C.byref(n)), "amp_sens_bgemm_workspace_bytes")
    return n.value


def amp_sens_bgemm(ops, fmts, d_out, workspace, stream=None):
    f, nf = _fmts(fmts)
    _check(lib().amp_sens_bgemm(_array(BgemmDesc, ops), len(ops), f, nf, _ptr(d_out),
                                _ptr(workspace), workspace.numel() * workspace.element_size(),
                                _stream(stream)), "amp_sens_bgemm")


def amp_sens_block_workspace_bytes(linears, bgemms, n_fmts):
    n = C.c_size_t()
    _check(lib().amp_sens_block_workspace_bytes(_array(LinearDesc, linears), len(linears),
                                                _array(BgemmDesc, bgemms), len(bgemms), int(n_fmts),
                                                C.byref(n)), "amp_sens_block_workspace_bytes")
    return n.value


def amp_sens_block(linears, bgemms, fmts, d_out, workspace, stream=None):
    """Linears and BGEMMs in one call; d_out [sum R of the linears + sum R of the BGEMMs, n_fmts, 4]."""
    f, nf = _fmts(fmts)
    _check(lib().amp_sens_block(_array(LinearDesc, linears), len(linears), _array(BgemmDesc, bgemms),
                                len(bgemms), f, nf, _ptr(d_out), _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream(stream)),
           "amp_sens_block")


STATIC_WORKSPACE_BYTES = 16 << 20


def amp_sens_block_static(linears, bgemms, fmts, d_out, stream=None):
    """amp_sens_block with the library's own fixed device array as workspace (no allocation anywhere)."""
    f, nf = _fmts(fmts)
    _check(lib().amp_sens_block_static(_array(LinearDesc, linears), len(linears), _array(BgemmDesc, bgemms),
                                       len(bgemms), f, nf, _ptr(d_out), _stream(stream)), "amp_sens_block_static")


def amp_absmax_scale_setup(tensors, fmts, d_amax, d_scale, d_inv, d_flags, workspace, stream=None):
    """The set-up half of amp_absmax_scale; returns the Plan for amp_run."""
    f, nf = _fmts(fmts)
    plan = Plan()
    _check(lib().amp_absmax_scale_setup(_array(Tensor, tensors), len(tensors), f, nf, _ptr(d_amax), _ptr(d_scale),
                                        _ptr(d_inv), _ptr(d_flags), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream(stream),
                                        C.byref(plan)), "amp_absmax_scale_setup")
    plan._keep = (tensors, d_amax, d_scale, d_inv, d_flags, workspace)
    return plan


def amp_absmax_scale_rows_setup(tensors, fmts, d_amax, d_scale, d_inv, d_flags, workspace, stream=None):
    f, nf = _fmts(fmts)
    plan = Plan()
    _check(lib().amp_absmax_scale_rows_setup(_array(Tensor, tensors), len(tensors), f, nf, _ptr(d_amax),
                                             _ptr(d_scale), _ptr(d_inv), _ptr(d_flags), _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _stream(stream),
                                             C.byref(plan)), "amp_absmax_scale_rows_setup")
    plan._keep = (tensors, d_amax, d_scale, d_inv, d_flags, workspace)
    return plan


def amp_sens_block_setup(linears, bgemms, fmts, d_out, workspace, flags=0, stream=None):
    """The set-up half of amp_sens_block (flags: PLAN_STREAM_WEIGHTS, plan_interleave(n)); returns the Plan."""
    f, nf = _fmts(fmts)
    plan = Plan()
    _check(lib().amp_sens_block_setup(_array(LinearDesc, linears), len(linears), _array(BgemmDesc, bgemms),
                                      len(bgemms), f, nf, _ptr(d_out), _ptr(workspace),
                                      workspace.numel() * workspace.element_size(), int(flags), _stream(stream),
                                      C.byref(plan)), "amp_sens_block_setup")
    plan._keep = (linears, bgemms, d_out, workspace)
    return plan


def amp_plan_limit_grid(plan, max_workgroups):
    _check(lib().amp_plan_limit_grid(C.byref(plan), int(max_workgroups)), "amp_plan_limit_grid")


def amp_run(plan, stream=None):
    _check(lib().amp_run(C.byref(plan), _stream(stream)), "amp_run")


def amp_loss_second_moment(losses):
    """E[g^2] over the samples' losses."""
    losses = np.ascontiguousarray(losses, dtype=np.float64)
    f = lib().amp_loss_second_moment
    f.restype = C.c_double
    f.argtypes = [C.c_void_p, C.c_int]
    return f(losses.ctypes.data_as(C.c_void_p), int(losses.size))


def amp_mse_budget(tau, mean_g2):
    """tau^2 E[g^2], the loss-MSE budget of eq. (ip)."""
    f = lib().amp_mse_budget
    f.restype = C.c_double
    f.argtypes = [C.c_double, C.c_double]
    return f(float(tau), float(mean_g2))


def amp_alpha(mantissa_bits):
    return lib().amp_alpha(int(mantissa_bits))


def amp_layer_loss_mse(sums, fmts):
    """sums: host float32 array [R, n_fmts, 4].  Returns (s_layer, d_model[n_fmts], d_measured[n_fmts])."""
    sums = np.ascontiguousarray(sums, dtype=np.float32)
    R = sums.shape[0]
    f, nf = _fmts(fmts)
    assert sums.shape == (R, nf, 4)
    s = C.c_double()
    dm = np.empty(nf, dtype=np.float64)
    de = np.empty(nf, dtype=np.float64)
    _check(lib().amp_layer_loss_mse(sums.ctypes.data_as(C.c_void_p), R, f, nf, C.byref(s),
                                    dm.ctypes.data_as(C.c_void_p), de.ctypes.data_as(C.c_void_p)),
           "amp_layer_loss_mse")
    return s.value, dm, de


def amp_group_tables(layer_mse, layer_gain):
    """layer_mse, layer_gain: [n_layers, F].  Returns (d[F**n_layers], c[F**n_layers])."""
    layer_mse = np.ascontiguousarray(layer_mse, dtype=np.float64)
    layer_gain = np.ascontiguousarray(layer_gain, dtype=np.float64)
    L, F = layer_mse.shape
    assert layer_gain.shape == (L, F)
    d = np.empty(F ** L, dtype=np.float64)
    c = np.empty(F ** L, dtype=np.float64)
    _check(lib().amp_group_tables(L, F, layer_mse.ctypes.data_as(C.c_void_p),
                                  layer_gain.ctypes.data_as(C.c_void_p),
                                  d.ctypes.data_as(C.c_void_p), c.ctypes.data_as(C.c_void_p)),
           "amp_group_tables")
    return d, c


def amp_select_subgraphs(n_choices, gain, mse, mse_budget):
    """Returns (choice[J], total_gain, total_mse); raises AmpError(ERR_INFEASIBLE) if nothing fits."""
    n_choices = np.ascontiguousarray(n_choices, dtype=np.int32)
    gain = np.ascontiguousarray(gain, dtype=np.float64)
    mse = np.ascontiguousarray(mse, dtype=np.float64)
    J = n_choices.size
    choice = np.zeros(max(J, 1), dtype=np.int32)
    tg, td = C.c_double(), C.c_double()
    _check(lib().amp_select_subgraphs(J, n_choices.ctypes.data_as(C.c_void_p),
                                      gain.ctypes.data_as(C.c_void_p),
                                      mse.ctypes.data_as(C.c_void_p), C.c_double(mse_budget),
                                      choice.ctypes.data_as(C.c_void_p), C.byref(tg), C.byref(td)),
           "amp_select_subgraphs")
    return choice[:J], tg.value, td.value


def amp_partition_sequential(n_vertices, edges, quantizable=None):
    """edges: iterable of (src, dst).  Returns (group_of[n_vertices] with -1 for dropped vertices, n_groups)."""
    edges = np.ascontiguousarray(np.asarray(list(edges), dtype=np.int32).reshape(-1, 2))
    src = np.ascontiguousarray(edges[:, 0])
    dst = np.ascontiguousarray(edges[:, 1])
    q = None if quantizable is None else np.ascontiguousarray(quantizable, dtype=np.uint8)
    group_of = np.full(n_vertices, -1, dtype=np.int32)
    ng = C.c_int32()
    _check(lib().amp_partition_sequential(int(n_vertices), int(src.size), src.ctypes.data_as(C.c_void_p),
                                          dst.ctypes.data_as(C.c_void_p),
                                          None if q is None else q.ctypes.data_as(C.c_void_p),
                                          group_of.ctypes.data_as(C.c_void_p), C.byref(ng)),
           "amp_partition_sequential")
    return group_of, ng.value


def amp_time_gain_macs(is_bgemm, N, C_, K, delta_t):
    f = lib().amp_time_gain_macs
    f.restype = C.c_double
    f.argtypes = [C.c_int, C.c_double, C.c_double, C.c_double, C.c_double]
    return f(int(is_bgemm), float(N), float(C_), float(K), float(delta_t))


def amp_memory_gain(is_bgemm, C_, K, delta_m):
    f = lib().amp_memory_gain
    f.restype = C.c_double
    f.argtypes = [C.c_int, C.c_double, C.c_double, C.c_double]
    return f(int(is_bgemm), float(C_), float(K), float(delta_m))


def amp_select_ordered(n_choices, gain, mse, mse_budget, order=None):
    """Prefix (order=None) / Random (order = a permutation) baselines.  Returns (choice, gain, mse)."""
    n_choices = np.ascontiguousarray(n_choices, dtype=np.int32)
    gain = np.ascontiguousarray(gain, dtype=np.float64)
    mse = np.ascontiguousarray(mse, dtype=np.float64)
    J = n_choices.size
    o = None if order is None else np.ascontiguousarray(order, dtype=np.int32)
    choice = np.zeros(max(J, 1), dtype=np.int32)
    tg, td = C.c_double(), C.c_double()
    _check(lib().amp_select_ordered(J, n_choices.ctypes.data_as(C.c_void_p), gain.ctypes.data_as(C.c_void_p),
                                    mse.ctypes.data_as(C.c_void_p), C.c_double(mse_budget),
                                    None if o is None else o.ctypes.data_as(C.c_void_p),
                                    choice.ctypes.data_as(C.c_void_p), C.byref(tg), C.byref(td)),
           "amp_select_ordered")
    return choice[:J], tg.value, td.value


def amp_profile_enable(max_launches):
    _check(lib().amp_profile_enable(int(max_launches)), "amp_profile_enable")


KERNEL_WEIGHTS = 0
KERNEL_STREAM = 16


def amp_profile_kinds(capacity):
    """Which kernel each recorded launch was (KERNEL_WEIGHTS + 0 / 1, KERNEL_STREAM + class); call before
    amp_profile_read."""
    kinds = np.zeros(max(capacity, 1), dtype=np.int32)
    n = C.c_int()
    _check(lib().amp_profile_kinds(kinds.ctypes.data_as(C.c_void_p), int(capacity), C.byref(n)), "amp_profile_kinds")
    return kinds[:n.value].copy()


def amp_profile_read(capacity):
    """(milliseconds, element pairs, bytes defined to be read) of every fused-kernel launch since the
    last read."""
    ms = np.zeros(max(capacity, 1), dtype=np.float32)
    pairs = np.zeros(max(capacity, 1), dtype=np.uint64)
    nbytes = np.zeros(max(capacity, 1), dtype=np.uint64)
    n = C.c_int()
    _check(lib().amp_profile_read(ms.ctypes.data_as(C.c_void_p), pairs.ctypes.data_as(C.c_void_p),
                                  nbytes.ctypes.data_as(C.c_void_p), int(capacity), C.byref(n)),
           "amp_profile_read")
    return ms[:n.value].copy(), pairs[:n.value].copy(), nbytes[:n.value].copy()


def amp_version():
    return lib().amp_version()
