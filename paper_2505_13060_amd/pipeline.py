"""One calibration pass over a Workload through the C-ABI: absmax + scales for every operand
buffer, then the fused sensitivity pass over all linears and all BGEMMs.

Marshalling only: descriptors are assembled here, outputs and workspaces are torch device
tensors allocated once; every number is produced by libampsens' kernels.
"""
import numpy as np
import torch

from . import (ROWS_COMPUTE0, ROWS_COMPUTE1, ROWS_COMPUTE_MAX_ROW_LEN, ROWS_OPERAND0, ROWS_OPERAND1, amp_absmax_rows_workspace_bytes, amp_absmax_scale,
               amp_absmax_scale_rows, amp_absmax_scale_rows_setup, amp_absmax_scale_setup,
               amp_absmax_workspace_bytes, amp_plan_limit_grid, amp_run, amp_sens_bgemm,
               amp_sens_bgemm_workspace_bytes, amp_sens_block, amp_sens_block_setup,
               amp_sens_block_workspace_bytes, amp_sens_linear, amp_sens_linear_workspace_bytes, bgemm_desc,
               causal, dense, linear_desc, rows_block, tensor)


def _layout(lay, cols=0):
    return dense(lay[1], cols) if lay[0] == "dense" else causal(lay[1], lay[2], lay[3])


def _row(t, i):
    return t[i]


class SensPass:
    """Holds descriptors, outputs and workspaces for one Workload resident on `device`.
    one_call: linears and BGEMMs go through amp_sens_block (one table, one set-up, one streaming
    launch for activations and BGEMM operands) instead of amp_sens_linear + amp_sens_bgemm.
    plan: the set-up of both calls (absmax, sensitivity block) is done once, here, on the current
    stream, and run() only replays the plans (kernel launches only); flags go to
    amp_sens_block_setup, grid_limit to amp_plan_limit_grid."""

    def __init__(self, workload, device, one_call=False, plan=False, flags=0, grid_limit=0, rule=0):
        """rule: 0, or SCALE_POW2: power-of-two scales from the absmax call, and the promise to the
        sensitivity call that goes with them (it then casts with the scaled FP8 conversions)."""
        self.plan = plan or flags != 0 or grid_limit != 0
        one_call = one_call or self.plan
        self.one_call = one_call
        self.w = workload
        self.device = device
        self.rule = rule
        self.fmts = [f | rule for f in workload.fmts]
        nf = len(self.fmts)
        nl, nb = len(workload.linears), len(workload.bgemms)
        self.tensors = []
        for op in workload.linears:
            self.tensors.append(tensor(op.x, dense(int(op.row_offsets[-1]) * op.C)))
            self.tensors.append(tensor(op.w, dense(op.K * op.C)))
        for op in workload.bgemms:
            self.tensors.append(tensor(op.x0, _layout(op.lay0), op.R))
            self.tensors.append(tensor(op.x1, _layout(op.lay1), op.R))
        nt = len(self.tensors)
        f32 = dict(device=device, dtype=torch.float32)
        self.d_amax = torch.zeros(max(nt, 1), **f32)
        self.d_scale = torch.zeros(max(nt, 1), nf, **f32)
        self.d_inv = torch.zeros(max(nt, 1), nf, **f32)
        self.d_flags = torch.zeros(max(nt, 1), device=device, dtype=torch.int32)

        self.lin_desc = []
        for k, op in enumerate(workload.linears):
            uniform = np.array_equal(op.row_offsets, np.arange(op.R + 1) * (op.row_offsets[1] if op.R else 0))
            self.lin_desc.append(linear_desc(
                op.x, op.dx, op.w, op.dw, op.C, op.K, op.R,
                self.d_scale[2 * k], self.d_inv[2 * k], self.d_scale[2 * k + 1], self.d_inv[2 * k + 1],
                tokens=int(op.row_offsets[1]) if (uniform and op.R) else 0,
                sample_row_offsets=None if uniform else op.row_offsets))
        self.bg_desc = []
        for k, op in enumerate(workload.bgemms):
            t0 = 2 * nl + 2 * k
            self.bg_desc.append(bgemm_desc(op.x0, op.dx0, _layout(op.lay0), op.x1, op.dx1,
                                           _layout(op.lay1), op.R, self.d_scale[t0], self.d_inv[t0],
                                           self.d_scale[t0 + 1], self.d_inv[t0 + 1]))
        self.lin_R = [op.R for op in workload.linears]
        self.bg_R = [op.R for op in workload.bgemms]
        nlr, nbr = sum(self.lin_R), sum(self.bg_R)
        self.d_out = torch.zeros(max(nlr + nbr, 1), nf, 4, **f32)      # the linears' block, then the BGEMMs'
        self.d_lin_out = self.d_out[:nlr]
        self.d_bg_out = self.d_out[nlr:nlr + nbr]

        def ws(nbytes):
            return torch.empty(max(nbytes, 256), device=device, dtype=torch.uint8)

        self.ws_abs = ws(amp_absmax_workspace_bytes(self.tensors))
        if one_call:
            self.ws_block = ws(amp_sens_block_workspace_bytes(self.lin_desc, self.bg_desc, nf))
        else:
            self.ws_lin = ws(amp_sens_linear_workspace_bytes(self.lin_desc, nf))
            self.ws_bg = ws(amp_sens_bgemm_workspace_bytes(self.bg_desc, nf))
        if self.plan:
            self.abs_plan = amp_absmax_scale_setup(self.tensors, self.fmts, self.d_amax, self.d_scale, self.d_inv,
                                                   self.d_flags, self.ws_abs)
            self.sens_plan = amp_sens_block_setup(self.lin_desc, self.bg_desc, self.fmts, self.d_out,
                                                  self.ws_block, flags)
            self.limit_grid(grid_limit)

    def limit_grid(self, max_workgroups):
        amp_plan_limit_grid(self.abs_plan, max_workgroups)
        amp_plan_limit_grid(self.sens_plan, max_workgroups)

    def absmax(self, stream=None):
        if self.plan:
            amp_run(self.abs_plan, stream)
            return
        amp_absmax_scale(self.tensors, self.fmts, self.d_amax, self.d_scale, self.d_inv, self.d_flags,
                         self.ws_abs, stream)

    def sens(self, stream=None):
        if self.plan:
            amp_run(self.sens_plan, stream)
            return
        if self.one_call:
            amp_sens_block(self.lin_desc, self.bg_desc, self.fmts, self.d_out, self.ws_block, stream)
            return
        if self.lin_desc:
            amp_sens_linear(self.lin_desc, self.fmts, self.d_lin_out, self.ws_lin, stream)
        if self.bg_desc:
            amp_sens_bgemm(self.bg_desc, self.fmts, self.d_bg_out, self.ws_bg, stream)

    def run(self, stream=None):
        """One pass of the whole device path; asynchronous."""
        self.absmax(stream)
        self.sens(stream)

    def results(self, scales=True):
        """Synchronise and copy the small outputs to the host (scales=False: the sums and flags only)."""
        torch.cuda.synchronize(self.device)
        lin = self.d_lin_out.cpu().numpy()
        bg = self.d_bg_out.cpu().numpy()
        lin_ops, bg_ops, o = [], [], 0
        for R in self.lin_R:
            lin_ops.append(lin[o:o + R])
            o += R
        o = 0
        for R in self.bg_R:
            bg_ops.append(bg[o:o + R])
            o += R
        out = dict(flags=self.d_flags.cpu().numpy(), linear=lin_ops, bgemm=bg_ops, pow2=self.rule != 0)
        if scales:
            out.update(amax=self.d_amax.cpu().numpy(), scale=self.d_scale.cpu().numpy(),
                       inv=self.d_inv.cpu().numpy())
        return out


class RowSensPass:
    """The same pass with one scale per row where asked for: per token for the activations of the
    linears (x_rows), per output channel for their weights (w_rows), per row of the BGEMM
    operands (bgemm_rows; a dense operand's row is its last dimension).  Operands left at one
    scale per tensor go through amp_absmax_scale as in SensPass."""

    def __init__(self, workload, device, x_rows=True, w_rows=True, bgemm_rows=True, one_call=False, plan=False,
                 flags=0, single_read=False, rule=0, block=0):
        """rule: 0 or SCALE_POW2 (power-of-two scales everywhere, as in SensPass).  block: 0, or the length
        of the 1 x block scale tiles every dense row is cut into (it must divide the row lengths it meets;
        causal rows keep one scale each).  single_read: the row scales of the activations and of the BGEMM operands are computed by the
        sensitivity pass itself (AMP_ROWS_COMPUTE0 / 1: every row is fetched once); only the weights'
        per-channel scales then come from amp_absmax_scale_rows."""
        self.single_read = single_read
        self.plan = plan or flags != 0
        one_call = one_call or self.plan
        self.one_call = one_call
        self.w, self.device, self.fmts = workload, device, [f | rule for f in workload.fmts]
        self.rule = rule
        nf = len(self.fmts)
        f32 = dict(device=device, dtype=torch.float32)
        self.block = int(block)

        def scale_len(cols):                         # elements of a dense row that share a scale
            if block:
                assert cols % block == 0, "the scale block must divide every dense row it is applied to"
                return block
            return cols

        def blocked(lay):
            return dense(lay.n_elems, scale_len(lay.cols)) if not lay.causal else lay

        per_tensor, per_row = [], []                 # (key, Tensor)
        for k, op in enumerate(workload.linears):
            rows = int(op.row_offsets[-1])
            (per_row if x_rows else per_tensor).append((("lin", k, 0), tensor(op.x, dense(rows * op.C, scale_len(op.C)))))
            (per_row if w_rows else per_tensor).append((("lin", k, 1), tensor(op.w, dense(op.K * op.C, scale_len(op.C)))))
        for k, op in enumerate(workload.bgemms):
            for side, (x, lay) in enumerate(((op.x0, op.lay0), (op.x1, op.lay1))):
                t = tensor(x, blocked(_layout(lay, x.shape[-1])), op.R)
                (per_row if bgemm_rows else per_tensor).append((("bg", k, side), t))
        # operands whose row scales the sensitivity pass computes itself: their tables sit behind the others'
        # (rows too long for the single-read pass, or not made of whole vectors, keep the two-pass form)
        self.computed = set(key for key, t in per_row if single_read and (key[0] == "bg" or key[2] == 0)
                            and t.layout.cols % 8 == 0 and t.layout.cols <= ROWS_COMPUTE_MAX_ROW_LEN)
        per_row = [kt for kt in per_row if kt[0] not in self.computed] + [kt for kt in per_row if kt[0] in self.computed]
        self.t_tensors = [t for _, t in per_tensor]
        self.r_tensors = [t for key, t in per_row if key not in self.computed]
        nt = max(len(self.t_tensors), 1)
        self.d_amax = torch.zeros(nt, **f32)
        self.d_scale = torch.zeros(nt, nf, **f32)
        self.d_inv = torch.zeros(nt, nf, **f32)
        self.d_flags = torch.zeros(nt, device=device, dtype=torch.int32)
        ws_rows, _ = amp_absmax_rows_workspace_bytes(self.r_tensors)
        n_rows = sum(amp_absmax_rows_workspace_bytes([t])[1] for _, t in per_row)
        self.n_rows = n_rows
        self.r_amax = torch.zeros(max(n_rows, 1), **f32)
        self.r_scale = torch.zeros(max(n_rows, 1), nf, **f32)
        self.r_inv = torch.zeros(max(n_rows, 1), nf, **f32)
        self.r_flags = torch.zeros(max(len(self.r_tensors), 1), device=device, dtype=torch.int32)
        # where each operand's scales start
        self.where = {}
        for i, (key, _) in enumerate(per_tensor):
            self.where[key] = ("tensor", i)
        base = 0
        for i, (key, t) in enumerate(per_row):
            _, rows = amp_absmax_rows_workspace_bytes([t])
            self.where[key] = ("rows", base, rows, i)
            base += rows

        def scales(key):
            w = self.where[key]
            if w[0] == "tensor":
                return self.d_scale[w[1]], self.d_inv[w[1]], 0
            return self.r_scale[w[1]:], self.r_inv[w[1]:], 1

        self.lin_desc, self.bg_desc = [], []
        for k, op in enumerate(workload.linears):
            uniform = np.array_equal(op.row_offsets, np.arange(op.R + 1) * (op.row_offsets[1] if op.R else 0))
            xs, xi, xr = scales(("lin", k, 0))
            ws_, wi, wr = scales(("lin", k, 1))
            self.lin_desc.append(linear_desc(
                op.x, op.dx, op.w, op.dw, op.C, op.K, op.R, xs, xi, ws_, wi,
                tokens=int(op.row_offsets[1]) if (uniform and op.R) else 0,
                sample_row_offsets=None if uniform else op.row_offsets,
                scale_rows=((ROWS_COMPUTE0 if ("lin", k, 0) in self.computed else ROWS_OPERAND0) if xr else 0) |
                           (ROWS_OPERAND1 if wr else 0) | (rows_block(block) if block and (xr or wr) else 0)))
        for k, op in enumerate(workload.bgemms):
            s0, i0, r0 = scales(("bg", k, 0))
            s1, i1, r1 = scales(("bg", k, 1))
            # a dense BGEMM operand says its scale blocks through its row length
            self.bg_desc.append(bgemm_desc(op.x0, op.dx0, blocked(_layout(op.lay0, op.x0.shape[-1])) if r0 else _layout(op.lay0, op.x0.shape[-1]),
                                           op.x1, op.dx1,
                                           blocked(_layout(op.lay1, op.x1.shape[-1])) if r1 else _layout(op.lay1, op.x1.shape[-1]),
                                           op.R, s0, i0, s1, i1,
                                           scale_rows=((ROWS_COMPUTE0 if ("bg", k, 0) in self.computed else ROWS_OPERAND0) if r0 else 0) |
                                                      ((ROWS_COMPUTE1 if ("bg", k, 1) in self.computed else ROWS_OPERAND1) if r1 else 0)))
        self.lin_R = [op.R for op in workload.linears]
        self.bg_R = [op.R for op in workload.bgemms]
        nlr, nbr = sum(self.lin_R), sum(self.bg_R)
        self.d_out = torch.zeros(max(nlr + nbr, 1), nf, 4, **f32)
        self.d_lin_out = self.d_out[:nlr]
        self.d_bg_out = self.d_out[nlr:nlr + nbr]

        def ws(nbytes):
            return torch.empty(max(nbytes, 256), device=device, dtype=torch.uint8)

        self.ws_abs = ws(amp_absmax_workspace_bytes(self.t_tensors))
        self.ws_rows = ws(ws_rows)
        if one_call:
            self.ws_block = ws(amp_sens_block_workspace_bytes(self.lin_desc, self.bg_desc, nf))
        else:
            self.ws_lin = ws(amp_sens_linear_workspace_bytes(self.lin_desc, nf))
            self.ws_bg = ws(amp_sens_bgemm_workspace_bytes(self.bg_desc, nf))
        if self.plan:
            self.abs_plan = amp_absmax_scale_setup(self.t_tensors, self.fmts, self.d_amax, self.d_scale, self.d_inv,
                                                   self.d_flags, self.ws_abs)
            self.rows_plan = amp_absmax_scale_rows_setup(self.r_tensors, self.fmts, self.r_amax, self.r_scale,
                                                         self.r_inv, self.r_flags, self.ws_rows)
            self.sens_plan = amp_sens_block_setup(self.lin_desc, self.bg_desc, self.fmts, self.d_out,
                                                  self.ws_block, flags)

    def absmax(self, stream=None):
        if self.plan:
            amp_run(self.abs_plan, stream)
            amp_run(self.rows_plan, stream)
            return
        if self.t_tensors:
            amp_absmax_scale(self.t_tensors, self.fmts, self.d_amax, self.d_scale, self.d_inv, self.d_flags,
                             self.ws_abs, stream)
        if self.r_tensors:
            amp_absmax_scale_rows(self.r_tensors, self.fmts, self.r_amax, self.r_scale, self.r_inv,
                                  self.r_flags, self.ws_rows, stream)

    def sens(self, stream=None):
        if self.plan:
            amp_run(self.sens_plan, stream)
            return
        if self.one_call:
            amp_sens_block(self.lin_desc, self.bg_desc, self.fmts, self.d_out, self.ws_block, stream)
            return
        if self.lin_desc:
            amp_sens_linear(self.lin_desc, self.fmts, self.d_lin_out, self.ws_lin, stream)
        if self.bg_desc:
            amp_sens_bgemm(self.bg_desc, self.fmts, self.d_bg_out, self.ws_bg, stream)

    def run(self, stream=None):
        self.absmax(stream)
        self.sens(stream)

    def results(self, scales=True):
        """scales=False leaves the per-row scale tables (12–20 bytes per row) on the device."""
        torch.cuda.synchronize(self.device)
        lin = self.d_lin_out.cpu().numpy()
        bg = self.d_bg_out.cpu().numpy()
        lin_ops, bg_ops, o = [], [], 0
        for R in self.lin_R:
            lin_ops.append(lin[o:o + R])
            o += R
        o = 0
        for R in self.bg_R:
            bg_ops.append(bg[o:o + R])
            o += R
        out = dict(flags=self.d_flags.cpu().numpy(), row_flags=self.r_flags.cpu().numpy(),
                   where=dict(self.where), computed=set(self.computed), linear=lin_ops, bgemm=bg_ops)
        if scales:
            out.update(amax=self.d_amax.cpu().numpy(), scale=self.d_scale.cpu().numpy(),
                       inv=self.d_inv.cpu().numpy(), row_amax=self.r_amax.cpu().numpy(),
                       row_scale=self.r_scale.cpu().numpy(), row_inv=self.r_inv.cpu().numpy())
        return out
