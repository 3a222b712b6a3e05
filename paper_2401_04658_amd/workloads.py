"""Seeded synthetic inputs for the benchmark configurations.

Holds no attention arithmetic: only shapes, seeds, value distributions and the
per-head decay schedule.  Both the GPU tests/benchmark and the CPU oracle's
callers draw their inputs here, so the two sides always see identical values.

Every tensor is drawn on the CPU with a seeded torch.Generator, in the order
Q, K, V, dO, as fp32 standard normals, scaled, then cast to the configuration's
storage dtype (bf16 values are what both sides consume; the oracle up-casts them
exactly).
"""
import math
from dataclasses import dataclass, field
from typing import Optional

import torch


def head_decay(heads: int) -> torch.Tensor:
    """lambda_h = exp(-2^(-8 (h+1) / H)), h = 0 .. H-1, as fp32."""
    h = torch.arange(1, heads + 1, dtype=torch.float64)
    return torch.exp(-torch.pow(torch.tensor(2.0, dtype=torch.float64), -8.0 * h / heads)).to(torch.float32)


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    heads: int
    seqlen: int
    head_dim: int
    dtype: torch.dtype
    seed: int
    backward: bool = True
    qk_scale: Optional[float] = None      # default 1/sqrt(d)
    v_scale: Optional[float] = None       # default 1/sqrt(d)
    fixed_lambda: Optional[float] = None  # one decay for all heads instead of the schedule

    @property
    def tokens(self) -> int:
        return self.batch * self.seqlen

    @property
    def token_heads(self) -> int:
        return self.batch * self.heads * self.seqlen

    def decay(self) -> torch.Tensor:
        if self.fixed_lambda is not None:
            return torch.full((self.heads,), self.fixed_lambda, dtype=torch.float32)
        return head_decay(self.heads)

    def tensors(self):
        """Returns dict with q, k, v, (d_o), lam on the CPU."""
        g = torch.Generator(device="cpu")
        g.manual_seed(self.seed)
        shape = (self.batch, self.heads, self.seqlen, self.head_dim)
        s_qk = self.qk_scale if self.qk_scale is not None else 1.0 / math.sqrt(self.head_dim)
        s_v = self.v_scale if self.v_scale is not None else 1.0 / math.sqrt(self.head_dim)
        out = {}
        for name, scale in (("q", s_qk), ("k", s_qk), ("v", s_v), ("d_o", s_v)):
            if name == "d_o" and not self.backward:
                break
            x = torch.randn(shape, generator=g, dtype=torch.float32)
            out[name] = (x * scale).to(self.dtype)
        out["lam"] = self.decay()
        return out


# The five configurations of the benchmark plan.
CONFIG1 = Workload("config1_fwd_fp32_n256_d64", 1, 1, 256, 64, torch.float32, seed=0, backward=False,
                   fixed_lambda=0.95)
CONFIG2 = Workload("config2_400M_layer_b4_h16_n2048_d64", 4, 16, 2048, 64, torch.bfloat16, seed=2)
CONFIG3 = tuple(
    Workload("config3_sweep_b%d_n%d_h16_d128" % (b, n), b, 16, n, 128, torch.bfloat16, seed=s)
    for (b, n, s) in ((64, 1024, 30), (16, 4096, 31), (4, 16384, 32), (1, 65536, 33))
)
CONFIG4 = Workload("config4_3B_layer_b2_h32_n16384_d128", 2, 32, 16384, 128, torch.bfloat16, seed=4,
                   v_scale=1.0)


@dataclass(frozen=True)
class DecodeWorkload:
    name: str = "config5_decode_b128_h32_d128"
    batch: int = 128
    heads: int = 32
    head_dim: int = 128
    steps: int = 1024
    seed: int = 5
    state_std: float = 0.1   # "N(0, 0.01)" read as variance 0.01

    def decay(self) -> torch.Tensor:
        return head_decay(self.heads)

    def generator(self) -> torch.Generator:
        g = torch.Generator(device="cpu")
        g.manual_seed(self.seed)
        return g

    def initial_state(self, g: torch.Generator) -> torch.Tensor:
        shape = (self.batch, self.heads, self.head_dim, self.head_dim)
        return torch.randn(shape, generator=g, dtype=torch.float32) * self.state_std

    def token(self, g: torch.Generator):
        """One step's q, k, v (bf16, [batch, heads, d]); call once per step, in order."""
        shape = (self.batch, self.heads, self.head_dim)
        s = 1.0 / math.sqrt(self.head_dim)
        return tuple((torch.randn(shape, generator=g, dtype=torch.float32) * s).to(torch.bfloat16) for _ in range(3))


CONFIG5 = DecodeWorkload()
