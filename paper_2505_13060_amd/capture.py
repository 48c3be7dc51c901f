"""Capture layer: hands the operands and loss gradients of a PyTorch model's quantisable
operations to libampsens, one calibration sample per forward/backward pass (step 2 of
Algorithm 1, App. A: the sensitivity of every layer is measured on the unquantised model from one
forward and one backward pass per sample; Sec. 2.2 defines z_l as the operands of op l and
z_l-dot as the loss gradient with respect to them).

Hook logic only: no FP8, no scales and no sums are computed here.  A sink receives, per sample,
the tensors of every op; the two library sinks turn them into descriptors and call the C-ABI.

  Capture(model, sink)             hooks every nn.Linear (or the named ones)
  cap.bgemm(name, a, b, causal_a)  call this instead of torch.matmul at an attention matmul
  cap.sample(loss_fn)              one forward/backward pass = one calibration sample

What "the gradient with respect to the operand of op l" means when a tensor feeds several ops
(q, k and v read the same hidden state): the perturbation of Sec. 2.2 is applied to the operand
as op l sees it, so each op gets the gradient that flows through it alone.  The hooks therefore
pass every op a private alias of its input and read the gradient of that alias.

The weight gradient of a sample is the module's weight.grad after the sample's backward pass
(gradients are cleared before each sample); a weight shared by several modules is not supported.
"""
from collections import OrderedDict

import numpy as np
import torch

from . import amp_loss_second_moment
from . import workloads as wl


class _Rec:
    __slots__ = ("kind", "name", "x", "dx", "w", "dw", "x1", "dx1", "causal", "module", "macs")

    def __init__(self, kind, name):
        self.kind, self.name = kind, name
        self.x = self.dx = self.w = self.dw = self.x1 = self.dx1 = self.module = None
        self.causal = False
        self.macs = 0.0


def _alias(t):
    """A tensor equal to t whose gradient is the part of t's gradient that flows through this use."""
    if t.requires_grad:
        return t.view_as(t)
    return t.detach().requires_grad_(True)


class Capture:
    def __init__(self, model, sink, linears=None):
        """linears: iterable of module names to hook (default: every torch.nn.Linear of `model`)."""
        self.model = model
        self.sink = sink
        self._recs = None
        self._handles = []
        wanted = None if linears is None else set(linears)
        self.linear_names = []
        for name, m in model.named_modules():
            if isinstance(m, torch.nn.Linear) and (wanted is None or name in wanted):
                self._handles.append(m.register_forward_pre_hook(self._pre_hook(name)))
                self.linear_names.append(name)
        if wanted is not None and wanted - set(self.linear_names):
            raise ValueError("not torch.nn.Linear modules of the model: %s" % sorted(wanted - set(self.linear_names)))

    def close(self):
        for h in self._handles:
            h.remove()
        self._handles = []

    # -- hooks ---------------------------------------------------------------------------------
    def _grad_into(self, rec, field):
        def hook(g):
            setattr(rec, field, g.detach())
        return hook

    def _pre_hook(self, name):
        def hook(module, args):
            if self._recs is None:
                return None                                    # outside sample(): leave the model alone
            if name in self._recs:
                raise RuntimeError("module %s ran twice in one sample; give each use its own module" % name)
            rec = _Rec("linear", name)
            x = _alias(args[0])
            x.register_hook(self._grad_into(rec, "dx"))
            rec.x, rec.w, rec.module = x.detach(), module.weight.detach(), module
            self._recs[name] = rec
            return (x,) + tuple(args[1:])
        return hook

    def bgemm(self, name, a, b, causal_a=False):
        """torch.matmul(a, b) whose operands are captured as BGEMM op `name` (eq. (bgemm_layer)).
        causal_a: a is [..., S, S'] with zeros above the diagonal i + (S' - S) that are not part
        of the operand (attention probabilities)."""
        if self._recs is None:
            return torch.matmul(a, b)
        if name in self._recs:
            raise RuntimeError("BGEMM %s ran twice in one sample" % name)
        rec = _Rec("bgemm", name)
        a_, b_ = _alias(a), _alias(b)
        a_.register_hook(self._grad_into(rec, "dx"))
        b_.register_hook(self._grad_into(rec, "dx1"))
        rec.x, rec.x1, rec.causal = a_.detach(), b_.detach(), bool(causal_a)
        rec.macs = float(a.numel()) * float(b.shape[-1])      # [.., M, K] x [.., K, N]: M*K*N per matrix
        self._recs[name] = rec
        return torch.matmul(a_, b_)

    # -- one calibration sample ------------------------------------------------------------------
    def sample(self, loss_fn):
        """Runs loss_fn() (a forward pass returning the scalar loss g^r), its backward pass, and
        hands every captured op to the sink.  Returns the loss value."""
        self.model.zero_grad(set_to_none=True)
        self._recs = OrderedDict()
        try:
            loss = loss_fn()
            loss.backward()
            recs = self._recs
        finally:
            self._recs = None
        for rec in recs.values():
            if rec.kind == "linear":
                g = rec.module.weight.grad
                if g is None:
                    raise RuntimeError("no weight gradient reached %s" % rec.name)
                rec.dw = g.detach().clone()
                rec.macs = float(rec.x.numel()) * float(rec.w.shape[0])
            if rec.dx is None or (rec.kind == "bgemm" and rec.dx1 is None):
                raise RuntimeError("no gradient reached an operand of %s" % rec.name)
        value = float(loss.detach())
        self.sink.add_sample(list(recs.values()), value)
        return value


# ---- sinks ---------------------------------------------------------------------------------------

class RecordingSink:
    """Keeps the captured tensors (for tests and inspection)."""

    def __init__(self):
        self.samples = []
        self.losses = []

    def add_sample(self, recs, loss):
        self.samples.append(recs)
        self.losses.append(loss)


def _bf16_2d(t, cols):
    return t.to(torch.bfloat16).reshape(-1, cols).contiguous()


def _ops_of(samples, fmts):
    """Stacks the samples' tensors of every op into the resident layout of the library:
    X, X-dot [sum_r tokens_r, C]; W [K, C]; W-dot [R, K, C]; BGEMM operands [R, ...]."""
    R = len(samples)
    linears, bgemms = [], []
    for i, first in enumerate(samples[0]):
        recs = [s[i] for s in samples]
        if any(r.name != first.name or r.kind != first.kind for r in recs):
            raise RuntimeError("samples ran different ops (%s)" % first.name)
        if first.kind == "linear":
            K, C_ = first.w.shape
            xs = [_bf16_2d(r.x, C_) for r in recs]
            offs = np.zeros(R + 1, dtype=np.int64)
            offs[1:] = np.cumsum([x.shape[0] for x in xs])
            linears.append(wl.LinearOp(first.name, torch.cat(xs), torch.cat([_bf16_2d(r.dx, C_) for r in recs]),
                                       first.w.to(torch.bfloat16).contiguous(),
                                       torch.stack([r.dw.to(torch.bfloat16).contiguous() for r in recs]),
                                       R, C_, K, offs))
        else:
            shapes = {(tuple(r.x.shape), tuple(r.x1.shape)) for r in recs}
            if len(shapes) != 1:
                raise RuntimeError("BGEMM %s: operand shapes differ between samples; capture such samples "
                                   "one by one (StreamSink)" % first.name)
            a = first.x
            if first.causal:
                rows, cols = a.shape[-2], a.shape[-1]
                lay0 = ("causal", a.numel() // (rows * cols), rows, cols)
            else:
                lay0 = ("dense", a.numel())
            stack = lambda ts: torch.stack([t.to(torch.bfloat16).contiguous() for t in ts])
            bgemms.append(wl.BgemmOp(first.name, stack([r.x for r in recs]), stack([r.dx for r in recs]), lay0,
                                     stack([r.x1 for r in recs]), stack([r.dx1 for r in recs]),
                                     ("dense", first.x1.numel()), R, macs=sum(r.macs for r in recs)))
    return wl.Workload("captured", list(fmts), linears, bgemms)


def _run(workload, device):
    from .pipeline import SensPass                              # loads the library: fails loudly without it
    p = SensPass(workload, device, one_call=True)
    p.run()
    res = p.results()
    if res["flags"].any():
        bad = [i for i, f in enumerate(res["flags"]) if f]
        raise FloatingPointError("non-finite values in captured operand buffers %s" % bad)
    out = OrderedDict()
    for k, op in enumerate(workload.linears):
        out[op.name] = res["linear"][k]
    for k, op in enumerate(workload.bgemms):
        out[op.name] = res["bgemm"][k]
    return out, res


class ResidentSink:
    """Keeps all samples, then runs the library once over the stacked tensors: one static
    per-tensor scale over all samples of an activation, W read once per batch of samples."""

    def __init__(self, fmts, device):
        self.fmts, self.device = list(fmts), device
        self.samples, self.losses = [], []
        self.raw = None                                         # the library's outputs incl. scales

    def add_sample(self, recs, loss):
        self.samples.append(recs)
        self.losses.append(loss)

    def workload(self):
        return _ops_of(self.samples, self.fmts)

    def finalize(self):
        """{op name: float32 sums [R, n_fmts, 4] = (E_0, A_0, E_1, A_1)}, E[g^2]."""
        out, self.raw = _run(self.workload(), self.device)
        return out, amp_loss_second_moment(self.losses)


class StreamSink:
    """Processes every sample as it is produced and keeps only the sums: activation scales are
    per sample (the scale of the sample's own tensor), W is read with every sample."""

    def __init__(self, fmts, device):
        self.fmts, self.device = list(fmts), device
        self.sums, self.losses = OrderedDict(), []
        self.raw = []                                           # per sample: the library's outputs incl. scales

    def add_sample(self, recs, loss):
        out, raw = _run(_ops_of([recs], self.fmts), self.device)
        for name, s in out.items():
            self.sums.setdefault(name, []).append(s[0])
        self.raw.append(raw)
        self.losses.append(loss)

    def finalize(self):
        return (OrderedDict((n, np.stack(v)) for n, v in self.sums.items()),
                amp_loss_second_moment(self.losses))
