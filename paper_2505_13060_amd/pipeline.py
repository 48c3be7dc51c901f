"""One calibration pass over a Workload through the C-ABI: absmax + scales for every operand
buffer, then the fused sensitivity pass over all linears and all BGEMMs.

Marshalling only: descriptors are assembled here, outputs and workspaces are torch device
tensors allocated once; every number is produced by libampsens' kernels.
"""
import numpy as np
import torch

from . import (amp_absmax_scale, amp_absmax_workspace_bytes, amp_sens_bgemm,
               amp_sens_bgemm_workspace_bytes, amp_sens_linear, amp_sens_linear_workspace_bytes,
               bgemm_desc, causal, dense, linear_desc, tensor)


def _layout(lay):
    return dense(lay[1]) if lay[0] == "dense" else causal(lay[1], lay[2], lay[3])


def _row(t, i):
    return t[i]


class SensPass:
    """Holds descriptors, outputs and workspaces for one Workload resident on `device`."""

    def __init__(self, workload, device):
        self.w = workload
        self.device = device
        self.fmts = list(workload.fmts)
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
        self.d_lin_out = torch.zeros(max(sum(self.lin_R), 1), nf, 4, **f32)
        self.d_bg_out = torch.zeros(max(sum(self.bg_R), 1), nf, 4, **f32)

        def ws(nbytes):
            return torch.empty(max(nbytes, 256), device=device, dtype=torch.uint8)

        self.ws_abs = ws(amp_absmax_workspace_bytes(self.tensors))
        self.ws_lin = ws(amp_sens_linear_workspace_bytes(self.lin_desc, nf))
        self.ws_bg = ws(amp_sens_bgemm_workspace_bytes(self.bg_desc, nf))

    def absmax(self, stream=None):
        amp_absmax_scale(self.tensors, self.fmts, self.d_amax, self.d_scale, self.d_inv, self.d_flags,
                         self.ws_abs, stream)

    def sens(self, stream=None):
        if self.lin_desc:
            amp_sens_linear(self.lin_desc, self.fmts, self.d_lin_out, self.ws_lin, stream)
        if self.bg_desc:
            amp_sens_bgemm(self.bg_desc, self.fmts, self.d_bg_out, self.ws_bg, stream)

    def run(self, stream=None):
        """One pass of the whole device path; asynchronous."""
        self.absmax(stream)
        self.sens(stream)

    def results(self):
        """Synchronise and copy the small outputs to the host."""
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
        return dict(amax=self.d_amax.cpu().numpy(), scale=self.d_scale.cpu().numpy(),
                    inv=self.d_inv.cpu().numpy(), flags=self.d_flags.cpu().numpy(),
                    linear=lin_ops, bgemm=bg_ops)
