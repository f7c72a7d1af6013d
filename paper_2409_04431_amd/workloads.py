"""Seeded synthetic inputs for the five benchmark configurations.

This module holds no attention arithmetic: it only draws tensors.  Both the GPU tests /
benchmark and the CPU oracle consume what it returns.  The draws stand in for the paper's
kernel benchmark on randomly initialised data (Appendix F.2): Q, K, V, dO are drawn in this
order in fp32 from torch.Generator('cpu').manual_seed(1000 + cfg) and then cast.
"""
import math
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Config:
    cfg: int
    B: int
    H: int
    N: int
    d: int
    dtype: torch.dtype
    causal: bool
    alibi: bool
    backward: bool
    qkv_scale: float      # multiplies the N(0,1) draws of Q, K, V
    v_uniform: bool       # V ~ U(-1,1) instead of N(0,1)

    @property
    def bias(self):
        return -math.log(self.N)

    @property
    def name(self):
        return (f"cfg{self.cfg}: B{self.B} H{self.H} N{self.N} d{self.d} "
                f"{'bf16' if self.dtype == torch.bfloat16 else 'fp32'}"
                f"{' causal' if self.causal else ''}{' alibi' if self.alibi else ''}")

    def fwd_flops(self):
        f = 4.0 * self.B * self.H * self.N * self.N * self.d
        return f * 0.5 if self.causal else f

    def bwd_flops(self):
        f = 10.0 * self.B * self.H * self.N * self.N * self.d
        return f * 0.5 if self.causal else f


CONFIGS = {
    1: Config(1, 1, 2, 256, 64, torch.float32, False, False, True, 1.0, False),
    2: Config(2, 4, 12, 1024, 64, torch.bfloat16, False, False, True, 64 ** -0.5, False),
    3: Config(3, 8, 16, 4096, 128, torch.bfloat16, True, False, True, 1.0, False),
    4: Config(4, 1, 32, 16384, 128, torch.bfloat16, True, True, True, 1.0, False),
    5: Config(5, 2, 8, 65536, 64, torch.bfloat16, False, False, False, 1.0, True),
}


def alibi_slopes(H):
    """Per-head slopes 2^(-8h/H), h = 1..H (geometric, ending at 2^-8)."""
    return torch.tensor([2.0 ** (-8.0 * (h + 1) / H) for h in range(H)], dtype=torch.float32)


def make_inputs(c, seed=None, shape=None):
    """Returns dict(q,k,v,dout[,slopes]) of CPU tensors in c.dtype (dout only if c.backward).
    `shape` overrides (B,H,N,d) for reduced-size parity cases with the same value recipe."""
    B, H, N, d = shape if shape is not None else (c.B, c.H, c.N, c.d)
    g = torch.Generator(device="cpu").manual_seed(1000 + c.cfg if seed is None else seed)
    out = {}
    out["q"] = (torch.randn(B, H, N, d, generator=g) * c.qkv_scale).to(c.dtype)
    out["k"] = (torch.randn(B, H, N, d, generator=g) * c.qkv_scale).to(c.dtype)
    if c.v_uniform:
        out["v"] = (torch.rand(B, H, N, d, generator=g) * 2.0 - 1.0).to(c.dtype)
    else:
        out["v"] = (torch.randn(B, H, N, d, generator=g) * c.qkv_scale).to(c.dtype)
    if c.backward:
        out["dout"] = torch.randn(B, H, N, d, generator=g).to(c.dtype)
    if c.alibi:
        out["slopes"] = alibi_slopes(H)
    return out
