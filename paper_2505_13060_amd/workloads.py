"""Seeded synthetic operand / gradient tensors with the shapes and value distributions of the
benchmark configurations (LLM decoder blocks).  Shared by the tests, the smoke check and the
benchmark; holds none of the method's arithmetic (no FP8, no scales, no sums): it only draws
bf16 tensors.  The same bytes go to the GPU library and, copied to the host, to the checker.

Recipes
  activation  N(0,1) (or Student-t, nu=4), a seeded subset of channels multiplied by 40
  weight      N(0, sigma^2)
  gradient    N(0, sigma_g^2) times a per-row lognormal(0, 0.5) factor (row = token for
              activations, output channel for weights)
  P           bf16 row-softmax of causally masked N(0, 2^2) logits, exact zeros above the diagonal;
              its gradient is zero there as well
Seeds: (1000*config + 16*block)*100 + tensor id, one torch.Generator per tensor.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def activation(seed, rows, C, device, outlier_channels=0, outlier_scale=40.0, student_nu=None):
    g = _gen(seed, device)
    x = torch.randn(rows, C, generator=g, device=device, dtype=torch.float32)
    if student_nu is not None:
        # t_nu = z / sqrt(chi2_nu / nu), chi2 from nu squared normals
        chi = torch.zeros(rows, C, device=device, dtype=torch.float32)
        for _ in range(int(student_nu)):
            chi += torch.randn(rows, C, generator=g, device=device, dtype=torch.float32) ** 2
        x = x / torch.sqrt(chi / float(student_nu))
    if outlier_channels > 0:
        idx = torch.randperm(C, generator=g, device=device)[:outlier_channels]
        x[:, idx] *= outlier_scale
    return x.to(torch.bfloat16)


def weight(seed, K, C, device, sigma=0.02):
    g = _gen(seed, device)
    return (torch.randn(K, C, generator=g, device=device, dtype=torch.float32) * sigma).to(torch.bfloat16)


def gradient(seed, rows, C, device, sigma=1e-3, lognormal_sigma=0.5, lead=()):
    """[*lead, rows, C] with a per-row scale."""
    g = _gen(seed, device)
    shape = tuple(lead) + (rows, C)
    z = torch.randn(*shape, generator=g, device=device, dtype=torch.float32) * sigma
    if lognormal_sigma > 0:
        s = torch.exp(torch.randn(*(tuple(lead) + (rows, 1)), generator=g, device=device,
                                  dtype=torch.float32) * lognormal_sigma)
        z = z * s
    return z.to(torch.bfloat16)


def causal_probs(seed, R, H, S, device):
    """P [R, H, S, S]: softmax over the causal prefix of N(0, 4) logits; zeros above the diagonal."""
    g = _gen(seed, device)
    out = torch.empty(R, H, S, S, device=device, dtype=torch.bfloat16)
    mask = torch.ones(S, S, device=device, dtype=torch.bool).tril()
    for r in range(R):
        logits = torch.randn(H, S, S, generator=g, device=device, dtype=torch.float32) * 2.0
        logits.masked_fill_(~mask, float("-inf"))
        out[r] = torch.softmax(logits, dim=-1).to(torch.bfloat16)
    return out


def causal_grad(seed, R, H, S, device, sigma=1e-3):
    d = gradient(seed, S, S, device, sigma=sigma, lead=(R, H))
    mask = torch.ones(S, S, device=device, dtype=torch.bool).tril()
    d.masked_fill_(~mask, 0.0)
    return d


@dataclass
class LinearOp:
    name: str
    x: torch.Tensor          # [rows_total, C]
    dx: torch.Tensor
    w: torch.Tensor          # [K, C]
    dw: torch.Tensor         # [R, K, C]
    R: int
    C: int
    K: int
    row_offsets: np.ndarray  # int64 [R+1]

    @property
    def macs(self):
        return float(int(self.row_offsets[-1]) * self.C * self.K)

    def pairs(self):
        return int(self.row_offsets[-1]) * self.C + self.R * self.K * self.C


@dataclass
class BgemmOp:
    name: str
    x0: torch.Tensor
    dx0: torch.Tensor
    lay0: tuple              # ("dense", n) or ("causal", batch, rows, cols)
    x1: torch.Tensor
    dx1: torch.Tensor
    lay1: tuple
    R: int
    macs: float = 0.0        # multiply-accumulates of the batched product, all samples

    @staticmethod
    def _valid(lay):
        if lay[0] == "dense":
            return lay[1]
        _, b, r, c = lay
        return b * sum(max(0, min(c, i + 1 + c - r)) for i in range(r))

    def pairs(self):
        return self.R * (self._valid(self.lay0) + self._valid(self.lay1))


@dataclass
class Workload:
    name: str
    fmts: List[int]
    linears: List[LinearOp] = field(default_factory=list)
    bgemms: List[BgemmOp] = field(default_factory=list)

    def pairs(self):
        return sum(o.pairs() for o in self.linears) + sum(o.pairs() for o in self.bgemms)


def _linear(name, seed, R, tokens, C, K, device, w_sigma=0.02, g_sigma=1e-3, outliers=0,
            student_nu=None, row_offsets=None):
    if row_offsets is None:
        row_offsets = np.arange(R + 1, dtype=np.int64) * tokens
    rows = int(row_offsets[-1])
    return LinearOp(name,
                    activation(seed, rows, C, device, outliers, 40.0, student_nu),
                    gradient(seed + 1, rows, C, device, g_sigma),
                    weight(seed + 2, K, C, device, w_sigma),
                    gradient(seed + 3, K, C, device, g_sigma, lead=(R,)),
                    R, C, K, np.asarray(row_offsets, dtype=np.int64))


def _attention(prefix, seed, R, Hq, Hkv, S, D, device, g_sigma=1e-3, outliers=0, student_nu=None):
    """QK^T (operands Q, K) and PV (operands P causal, V)."""
    def act(s, H):
        return activation(s, R * H * S, D, device, outliers, 40.0, student_nu).view(R, H, S, D)

    def grad(s, H):
        return gradient(s, S, D, device, g_sigma, lead=(R, H))

    qk = BgemmOp(prefix + "qk_matmul", act(seed, Hq), grad(seed + 1, Hq), ("dense", Hq * S * D),
                 act(seed + 2, Hkv), grad(seed + 3, Hkv), ("dense", Hkv * S * D), R,
                 float(R * Hq * S * S * D))
    pv = BgemmOp(prefix + "av_matmul", causal_probs(seed + 4, R, Hq, S, device),
                 causal_grad(seed + 5, R, Hq, S, device, g_sigma), ("causal", Hq, S, S),
                 act(seed + 6, Hkv), grad(seed + 7, Hkv), ("dense", Hkv * S * D), R,
                 float(R * Hq * S * S * D))
    return [qk, pv]


def config0(device, seed_base=0):
    """One linear layer, E4M3 only: X [4*256, 1024] with 8 outlier channels, W [1024, 1024]."""
    return Workload("config0", [0], [_linear("linear", seed_base, 4, 256, 1024, 1024, device, outliers=8)])


def decoder_block(name, cfg_id, device, R, S, hidden, ffn, Hq, Hkv, D, fmts, block=0, outlier_frac=0.01,
                  w_sigma=0.02, g_sigma=1e-3, student_nu=None):
    """Seven linears and two BGEMMs of one Llama-shaped decoder block."""
    sb = 1000 * cfg_id + 16 * block
    out = max(1, int(round(outlier_frac * hidden))) if outlier_frac > 0 else 0
    kw = dict(w_sigma=w_sigma, g_sigma=g_sigma, student_nu=student_nu)
    lin = [
        _linear("q_proj", sb * 100 + 0, R, S, hidden, Hq * D, device, outliers=out, **kw),
        _linear("k_proj", sb * 100 + 4, R, S, hidden, Hkv * D, device, outliers=out, **kw),
        _linear("v_proj", sb * 100 + 8, R, S, hidden, Hkv * D, device, outliers=out, **kw),
        _linear("o_proj", sb * 100 + 12, R, S, Hq * D, hidden, device, outliers=out, **kw),
        _linear("gate_proj", sb * 100 + 16, R, S, hidden, ffn, device, outliers=out, **kw),
        _linear("up_proj", sb * 100 + 20, R, S, hidden, ffn, device, outliers=out, **kw),
        _linear("down_proj", sb * 100 + 24, R, S, ffn, hidden, device,
                outliers=max(1, int(round(outlier_frac * ffn))) if outlier_frac > 0 else 0, **kw),
    ]
    bg = _attention("", sb * 100 + 28, R, Hq, Hkv, S, D, device, g_sigma=g_sigma,
                    outliers=max(1, int(round(outlier_frac * D))) if outlier_frac > 0 else 0,
                    student_nu=student_nu)
    return Workload(name, list(fmts), lin, bg)


def config1(device, R=8, S=2048, hidden=4096, ffn=11008, H=32, D=128, block=0, cfg_id=1):
    """One Llama-7B-shaped decoder block; E4M3 and E5M2."""
    return decoder_block("config1", cfg_id, device, R, S, hidden, ffn, H, H, D, [0, 1], block=block)


def config2_block(device, block, R=16, S=2048, hidden=4096, ffn=11008, H=32, D=128):
    """Block `block` of the 32-block 7B-shaped sweep (same shapes as config 1, R = 16)."""
    w = decoder_block("config2", 2, device, R, S, hidden, ffn, H, H, D, [0, 1], block=block)
    w.name = "config2/block%d" % block
    return w


def config3(device, R=8, S=4096, hidden=8192, ffn=28672, Hq=64, Hkv=8, D=128):
    """70B-shaped block, GQA, Student-t(4) activations, E4M3 only."""
    return decoder_block("config3", 3, device, R, S, hidden, ffn, Hq, Hkv, D, [0], outlier_frac=0.0,
                         w_sigma=0.015, g_sigma=5e-4, student_nu=4)


def config4(device, R=32, experts=64, C=4096, K=1408, tok_lo=16, tok_hi=512, n_bgemm=24, S=512,
            H=32, D=128):
    """Ragged: expert linears with a token count drawn per (expert, sample), plus small BGEMMs."""
    rng = np.random.default_rng(4000)
    lin = []
    for e in range(experts):
        counts = rng.integers(tok_lo, tok_hi + 1, R)
        off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
        lin.append(_linear("expert%d" % e, 400000 + 8 * e, R, 0, C, K, device,
                           outliers=max(1, int(round(0.01 * C))), row_offsets=off))
    bg = []
    for b in range(n_bgemm // 2):
        bg += _attention("l%d." % b, 450000 + 16 * b, R, H, H, S, D, device, outliers=1)
    return Workload("config4", [0, 1], lin, bg)


def to_bits(t: Optional[torch.Tensor]):
    """bf16 tensor -> numpy uint16 array on the host (same bytes)."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
