"""Seeded synthetic KV-cache workloads (input generation only).

This module holds none of the method's arithmetic: it only draws the fp16 K, V and q
tensors that stand in for the paper's OPT activations (Sec. 3.1 analyses OPT-6.7B keys
and values; Sec. 4.3 generates from wikitext-2 prompts -- neither the weights nor the
dataset are available, so shapes follow OPT's real head geometry and values follow the
distributions below).  Both the GPU tests/bench and the CPU oracle tests take their
inputs from here; the oracle always receives a copy of the very same fp16 bits.

Recipe (fixed draw order K, V, q from one seeded torch.Generator on the target device):
  K[b,h,t,d] = base[b,h,t,d] * chan[h,d]
      base ~ N(0,1)                              ("normal")
           ~ Student-t(5) / sqrt(5/3)  (unit var) ("student_t5")
      chan ~ LogNormal(0, 0.5), drawn once per tensor; `n_out` distinct channels per
      head (uniformly chosen) are multiplied by 10
  V[b,h,t,d] ~ N(0,1)
  q[b,h,d]   ~ N(0,1) / sqrt(D)                  (so softmax_scale = 1)
All values are drawn in fp32 and cast to fp16 with round-to-nearest-even.
"""
from __future__ import annotations

import dataclasses
import math

import torch


@dataclasses.dataclass(frozen=True)
class KVConfig:
    name: str
    B: int
    H: int
    D: int
    S: int                  # prefill / cached tokens
    decode_steps: int = 1   # tokens appended after prefill (cap = S + decode_steps when > 1)
    n_out: int = 0          # outlier channels per head in K
    k_dist: str = "normal"  # "normal" | "student_t5"
    bits: int = 4
    block: int = 64
    seed: int = 0

    @property
    def cap_tokens(self) -> int:
        return self.S + (self.decode_steps if self.decode_steps > 1 else 0)

    def with_(self, **kw) -> "KVConfig":
        return dataclasses.replace(self, **kw)


# The five benchmark configurations (OPT head geometries).
C1 = KVConfig("C1-opt125m", B=1, H=12, D=64, S=512, n_out=2)
C2 = KVConfig("C2-opt1.3b", B=8, H=32, D=64, S=2048, decode_steps=128, n_out=2)
C3 = KVConfig("C3-opt6.7b", B=32, H=32, D=128, S=2048, n_out=4)
C4 = KVConfig("C4-opt6.7b-long", B=1, H=32, D=128, S=32768, n_out=4)
C5 = KVConfig("C5-opt30b", B=16, H=56, D=128, S=16384, n_out=0, k_dist="student_t5")
CONFIGS = {c.name.split("-")[0]: c for c in (C1, C2, C3, C4, C5)}


def make_generator(cfg: KVConfig, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(cfg.seed)
    return g


def _channel_scales(cfg: KVConfig, device, g) -> torch.Tensor:
    chan = torch.exp(0.5 * torch.randn(cfg.H, cfg.D, device=device, generator=g, dtype=torch.float32))
    if cfg.n_out > 0:
        order = torch.rand(cfg.H, cfg.D, device=device, generator=g).argsort(dim=1)
        idx = order[:, : cfg.n_out]
        boost = torch.ones(cfg.H, cfg.D, device=device, dtype=torch.float32)
        boost.scatter_(1, idx, 10.0)
        chan = chan * boost
    return chan


def _base(cfg: KVConfig, shape, device, g) -> torch.Tensor:
    z = torch.randn(shape, device=device, generator=g, dtype=torch.float32)
    if cfg.k_dist == "normal":
        return z
    if cfg.k_dist == "student_t5":
        chi2 = torch.zeros(shape, device=device, dtype=torch.float32)
        for _ in range(5):
            chi2 += torch.randn(shape, device=device, generator=g, dtype=torch.float32) ** 2
        return z / torch.sqrt(chi2 / 5.0) / math.sqrt(5.0 / 3.0)
    raise ValueError(cfg.k_dist)


def make_kv(cfg: KVConfig, device, g: torch.Generator, n_tokens: int | None = None):
    """-> (K, V) fp16 [B, H, n_tokens, D] contiguous; K first, then V (one batch row at a time)."""
    n = cfg.S if n_tokens is None else n_tokens
    K = torch.empty(cfg.B, cfg.H, n, cfg.D, device=device, dtype=torch.float16)
    V = torch.empty_like(K)
    chan = _channel_scales(cfg, device, g)
    for b in range(cfg.B):
        K[b] = (_base(cfg, (cfg.H, n, cfg.D), device, g) * chan[:, None, :]).to(torch.float16)
    for b in range(cfg.B):
        V[b] = torch.randn(cfg.H, n, cfg.D, device=device, generator=g, dtype=torch.float32).to(torch.float16)
    return K, V


def make_q(cfg: KVConfig, device, g: torch.Generator) -> torch.Tensor:
    """-> q fp16 [B, H, D] ~ N(0,1)/sqrt(D)."""
    q = torch.randn(cfg.B, cfg.H, cfg.D, device=device, generator=g, dtype=torch.float32)
    return (q / math.sqrt(cfg.D)).to(torch.float16)


# ----------------------------------------------------------------- byte accounting
def fp16_kv_bytes(layers: int, hidden: int, batch: int, seq: int) -> int:
    """Bytes of an fp16 KV cache: K and V, 2 bytes each, per layer, hidden unit, sequence
    position and batch row (the paper's Sec. 1 example: OPT-175B, batch 64, seq 8192)."""
    return 2 * layers * hidden * 2 * batch * seq


def quantize_bytes_per_element(bits: int, block: int) -> float:
    """Algorithmic HBM bytes per quantized element: fp16 read + packed code + share of the fp16 scale."""
    return 2.0 + bits / 8.0 + 2.0 / block


def decode_bytes_per_token_head(D: int, bits: int, block: int) -> int:
    """Algorithmic HBM bytes read per cached token of one head (K and V codes and scales)."""
    return 2 * (D * bits // 8 + 2 * (D // block))
