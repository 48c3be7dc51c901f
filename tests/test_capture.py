"""Capture layer: the hooks deliver, per op and per sample, the operands and the loss gradients with
respect to them (Sec. 2.2: z_l and z_l-dot; step 2 of Algorithm 1).  CPU tests check the hook logic
against autograd and against the first-order expansion of the loss the statistic is built on; the
GPU tests run the library on the captured tensors and compare with the oracle."""
import os
import sys

import numpy as np
import pytest
import torch

sys.path.insert(0, os.path.dirname(__file__))
from tiny_model import TinyLlama  # noqa: E402

from paper_2505_13060_amd import capture as cp  # noqa: E402


def make(dtype=torch.float64, device="cpu", **kw):
    m = TinyLlama(**kw).to(dtype).to(device)
    sink = cp.RecordingSink()
    cap = cp.Capture(m, sink)
    m.mm = cap.bgemm
    return m, cap, sink


def tokens(seed, n=24, vocab=128, device="cpu"):
    g = torch.Generator().manual_seed(seed)
    return torch.randint(0, vocab, (n,), generator=g).to(device)


def test_every_op_is_captured_once_per_sample():
    m, cap, sink = make()
    for s in range(3):
        cap.sample(lambda: m.loss(tokens(s)))
    assert len(sink.samples) == 3
    names = [r.name for r in sink.samples[0]]
    want = []
    for b in range(2):
        want += ["blocks.%d.%s" % (b, n) for n in ("q_proj", "k_proj", "v_proj", "qk", "pv", "o_proj",
                                                   "gate_proj", "up_proj", "down_proj")]
    assert names == want + ["head"]
    for recs in sink.samples:
        for r in recs:
            assert r.dx.shape == r.x.shape
            if r.kind == "linear":
                assert r.dw.shape == r.w.shape
            else:
                assert r.dx1.shape == r.x1.shape


def test_loss_and_model_output_unchanged_by_the_hooks():
    m, cap, sink = make()
    t = tokens(5)
    plain = TinyLlama().to(torch.float64)
    assert float(plain.loss(t).detach()) == pytest.approx(cap.sample(lambda: m.loss(t)), rel=1e-13)
    # outside sample() the hooks are inert
    assert float(m.loss(t).detach()) == pytest.approx(float(plain.loss(t).detach()), rel=1e-13)


def test_weight_gradients_are_the_autograd_gradients_of_that_sample():
    m, cap, sink = make()
    for s in range(2):
        cap.sample(lambda: m.loss(tokens(10 + s)))
    ref = TinyLlama().to(torch.float64)
    for s in range(2):
        ref.zero_grad()
        ref.loss(tokens(10 + s)).backward()
        grads = dict((n, p.grad) for n, p in ref.named_parameters())
        for r in sink.samples[s]:
            if r.kind == "linear":
                assert torch.allclose(r.dw, grads[r.name + ".weight"], rtol=1e-12, atol=0), r.name


def test_input_gradient_is_the_part_through_that_op_only():
    """q, k and v read the same tensor: their three gradients differ and add up to the gradient of the
    shared tensor; each equals y-dot W of its own op."""
    m, cap, sink = make()
    cap.sample(lambda: m.loss(tokens(3)))
    recs = {r.name: r for r in sink.samples[0]}
    q, k, v = recs["blocks.1.q_proj"], recs["blocks.1.k_proj"], recs["blocks.1.v_proj"]
    assert torch.equal(q.x, k.x) and torch.equal(q.x, v.x)
    assert not torch.allclose(q.dx, k.dx)
    # independent computation: gradient with respect to the shared normalised hidden state
    ref = TinyLlama().to(torch.float64)
    keep = {}
    def keep_output(mod, args, out):
        out.retain_grad()
        keep["h"] = out

    h = ref.blocks[1].n1.register_forward_hook(keep_output)
    ref.loss(tokens(3)).backward()
    h.remove()
    assert torch.allclose(q.dx + k.dx + v.dx, keep["h"].grad, rtol=1e-10, atol=1e-18)


def test_first_order_expansion_of_the_loss():
    """Sec. 2.2 expands the loss to first order in the perturbation of z_l: perturbing one op's
    operand by eps*delta changes the loss by eps*<z-dot, delta> + O(eps^2).  Checked for a weight,
    for a linear's input and for both operands of a BGEMM, by re-running the model with the
    perturbation applied at that op only."""
    m, cap, sink = make()
    t = tokens(8)
    base = cap.sample(lambda: m.loss(t))
    recs = {r.name: r for r in sink.samples[0]}
    g = torch.Generator().manual_seed(1)
    eps = 1e-6

    def perturbed_loss(op, field, delta):
        ref = TinyLlama().to(torch.float64)
        if field == "w":
            with torch.no_grad():
                dict(ref.named_modules())[op].weight += eps * delta
        elif field == "x":
            dict(ref.named_modules())[op].register_forward_pre_hook(lambda mod, a: (a[0] + eps * delta,))
        else:
            def mm(name, a, b, causal_a):
                if name == op:
                    a, b = (a + eps * delta, b) if field == "a" else (a, b + eps * delta)
                return torch.matmul(a, b)
            ref.mm = mm
        return float(ref.loss(t).detach())

    cases = [("blocks.0.gate_proj", "w", "dw", "w"), ("blocks.1.k_proj", "x", "dx", "x"),
             ("blocks.0.qk", "a", "dx", "x"), ("blocks.0.qk", "b", "dx1", "x1"),
             ("blocks.1.pv", "a", "dx", "x"), ("blocks.1.pv", "b", "dx1", "x1")]
    for op, field, gname, xname in cases:
        r = recs[op]
        delta = torch.randn(getattr(r, xname).shape, generator=g, dtype=torch.float64)
        predicted = eps * float((getattr(r, gname) * delta).sum())
        actual = perturbed_loss(op, field, delta) - base
        assert actual == pytest.approx(predicted, rel=2e-3, abs=1e-14), (op, field)


def test_stacking_into_the_resident_layout():
    m, cap, sink = make(dtype=torch.bfloat16)
    lens = [24, 17, 30]
    for s, n in enumerate(lens):
        cap.sample(lambda: m.loss(tokens(s, n=n)))
    lin_only = [[r for r in recs if r.kind == "linear"] for recs in sink.samples]
    w = cp._ops_of(lin_only, [0, 1])
    assert [op.name for op in w.linears][:3] == ["blocks.0.q_proj", "blocks.0.k_proj", "blocks.0.v_proj"]
    op = w.linears[0]
    assert op.R == 3 and list(op.row_offsets) == [0, 23, 39, 68]
    assert op.x.shape == (68, 64) and op.dx.shape == (68, 64) and op.dw.shape == (3, 64, 64)
    assert torch.equal(op.x[23:39], sink.samples[1][0].x.reshape(-1, 64))
    assert torch.equal(op.dw[2], sink.samples[2][0].dw)
    # BGEMM operands of different sequence lengths cannot be stacked
    with pytest.raises(RuntimeError):
        cp._ops_of(sink.samples, [0, 1])
    # equal lengths: causal layout for P
    m2, cap2, sink2 = make(dtype=torch.bfloat16)
    for s in range(2):
        cap2.sample(lambda: m2.loss(tokens(s, n=21)))
    w2 = cp._ops_of(sink2.samples, [0])
    pv = [b for b in w2.bgemms if b.name == "blocks.0.pv"][0]
    assert pv.lay0 == ("causal", 4, 20, 20) and pv.lay1 == ("dense", 4 * 20 * 16)
    assert pv.x0.shape == (2, 4, 20, 20) and pv.R == 2
    assert float(pv.x0[0].float().triu(1).abs().max()) == 0.0


def test_capture_refuses_reuse_and_missing_modules():
    m = TinyLlama().to(torch.float64)
    with pytest.raises(ValueError):
        cp.Capture(m, cp.RecordingSink(), linears=["blocks.0.n1"])
    cap = cp.Capture(m, cp.RecordingSink(), linears=["blocks.0.q_proj"])
    assert cap.linear_names == ["blocks.0.q_proj"]
    x = torch.zeros(4, 64, dtype=torch.float64)

    def twice():
        return (m.blocks[0].q_proj(x) + m.blocks[0].q_proj(x)).sum()
    with pytest.raises(RuntimeError):
        cap.sample(twice)
    cap.close()


# ---- GPU: the library on captured tensors against the oracle ------------------------------------

@pytest.mark.gpu
@pytest.mark.parametrize("mode", ["resident", "stream"])
def test_gpu_captured_model_matches_oracle(mode):
    import parity
    from paper_2505_13060_amd import E4M3, E5M2
    dev = "cuda:0"
    fmts = [E4M3, E5M2]
    m = TinyLlama(vocab=256, d=128, heads=4, ffn=352, layers=2).to(torch.bfloat16).to(dev)
    rec = cp.RecordingSink()
    lib_sink = cp.ResidentSink(fmts, dev) if mode == "resident" else cp.StreamSink(fmts, dev)

    class Tee:
        def add_sample(self, recs, loss):
            rec.add_sample(recs, loss)
            lib_sink.add_sample(recs, loss)

    cap = cp.Capture(m, Tee())
    m.mm = cap.bgemm
    R = 3
    for s in range(R):
        print("capture sample", s, mode, flush=True)
        cap.sample(lambda: m.loss(tokens(40 + s, n=97, vocab=256, device=dev)))
    sums, g2 = lib_sink.finalize()
    assert g2 == pytest.approx(float(np.mean(np.square(rec.losses))))
    assert len(sums) == 2 * 9 + 1
    # the oracle on the very same bytes, copied to the host: scales bit for bit, sums to 1e-4
    if mode == "resident":
        parity.check_workload(cp._ops_of(rec.samples, fmts), lib_sink.raw)
        for name, v in sums.items():
            assert v.shape == (R, 2, 4), name
    else:
        for s in range(R):
            w = cp._ops_of([rec.samples[s]], fmts)
            parity.check_workload(w, lib_sink.raw[s])
            for k, op in enumerate(w.linears):
                assert np.array_equal(sums[op.name][s], lib_sink.raw[s]["linear"][k][0])
