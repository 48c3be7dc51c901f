"""A small randomly initialised Llama-shaped decoder (RMSNorm, causal multi-head attention, SwiGLU)
for the capture-layer tests.  The two attention matmuls go through `mm(name, a, b, causal_a)` so
that a capture object can see them; by default that is torch.matmul."""
import math

import torch
from torch import nn


def wide(t):
    """At least fp32 (bf16 models do their norms, softmax and loss in fp32; fp64 stays fp64)."""
    return t.to(torch.promote_types(t.dtype, torch.float32))


class RMSNorm(nn.Module):
    def __init__(self, d):
        super().__init__()
        self.g = nn.Parameter(torch.ones(d))

    def forward(self, x):
        v = wide(x).pow(2).mean(-1, keepdim=True)
        return (wide(x) * torch.rsqrt(v + 1e-5)).to(x.dtype) * self.g


class Block(nn.Module):
    def __init__(self, idx, d, heads, ffn):
        super().__init__()
        self.idx, self.h = idx, heads
        self.n1, self.n2 = RMSNorm(d), RMSNorm(d)
        self.q_proj, self.k_proj, self.v_proj, self.o_proj = (nn.Linear(d, d, bias=False) for _ in range(4))
        self.gate_proj, self.up_proj = nn.Linear(d, ffn, bias=False), nn.Linear(d, ffn, bias=False)
        self.down_proj = nn.Linear(ffn, d, bias=False)

    def forward(self, x, mm):
        S, d = x.shape
        h = self.n1(x)
        split = lambda t: t.view(S, self.h, d // self.h).transpose(0, 1)        # [H, S, D]
        q, k, v = split(self.q_proj(h)), split(self.k_proj(h)), split(self.v_proj(h))
        logits = mm("blocks.%d.qk" % self.idx, q, k.transpose(-1, -2), False) / math.sqrt(d // self.h)
        mask = torch.ones(S, S, dtype=torch.bool, device=x.device).tril()
        p = torch.softmax(wide(logits).masked_fill(~mask, float("-inf")), dim=-1).to(x.dtype)
        a = mm("blocks.%d.pv" % self.idx, p, v, True).transpose(0, 1).reshape(S, d)
        x = x + self.o_proj(a)
        h = self.n2(x)
        return x + self.down_proj(torch.nn.functional.silu(self.gate_proj(h)) * self.up_proj(h))


class TinyLlama(nn.Module):
    def __init__(self, vocab=128, d=64, heads=4, ffn=160, layers=2, seed=0):
        super().__init__()
        torch.manual_seed(seed)
        self.emb = nn.Embedding(vocab, d)
        self.blocks = nn.ModuleList(Block(i, d, heads, ffn) for i in range(layers))
        self.norm = RMSNorm(d)
        self.head = nn.Linear(d, vocab, bias=False)
        self.mm = lambda name, a, b, causal_a: torch.matmul(a, b)

    def loss(self, tokens):
        """Next-token cross entropy of one sequence (1-D LongTensor)."""
        x = self.emb(tokens[:-1])
        for b in self.blocks:
            x = b(x, self.mm)
        logits = wide(self.head(self.norm(x)))
        return torch.nn.functional.cross_entropy(logits, tokens[1:])
