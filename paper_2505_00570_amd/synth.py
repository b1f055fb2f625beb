"""Seeded synthetic KV tensors shaped like the paper's workloads (plumbing for tests and bench).

This module holds none of the compression arithmetic: it only draws random, low-frequency
dominated K and V states (the property Sec. 3.1 reports for LLaMA KV states) with the shapes of
Sec. 4.1, so that the HIP path and the CPU oracle can be fed identical bits.

  K : AR(1) per channel (rho 0.9), rotated RoPE-style over channel pairs (i, i + d/2) by
      angle p * base**(-2i/d) at absolute position p, 4 outlier channels per head scaled x8.
  V : AR(1) per channel (rho 0.8).
  tiny : AR(1) rho 0.95 plus N(0, 0.1^2) noise, fp32.
  q : decode queries, i.i.d. N(0, 0.5^2) (attention logits of a few units, as in trained models).

AR(1): a_0 = e_0 / sqrt(1 - rho^2), a_t = rho a_{t-1} + e_t, e ~ N(0, 1); the state is carried
across chunks so a stream of chunks is one long stationary sequence.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    batch: int
    n_heads: int          # KV heads
    head_dim: int
    window: int
    n_sink: int
    retain_ratio: float
    dtype: torch.dtype
    total_tokens: int     # tokens streamed through the cache
    rope_base: float = 10000.0
    rho_k: float = 0.9
    rho_v: float = 0.8
    n_q_heads: int = 0    # query heads (0: same as n_heads, i.e. multi-head attention)

    @property
    def q_heads(self) -> int:
        return self.n_q_heads or self.n_heads


WORKLOADS = {
    # the five benchmark configurations
    "tiny": Workload("tiny", 1, 1, 1, 64, 512, 4, 0.5, torch.float32, 512, rho_k=0.95, rho_v=0.95),
    "llama2_7b_layer": Workload("llama2_7b_layer", 1, 1, 32, 128, 4096, 4, 0.5, torch.bfloat16, 4096),
    "llama2_7b_32k": Workload("llama2_7b_32k", 32, 1, 32, 128, 4096, 4, 0.5, torch.bfloat16, 32768),
    "llama3_8b_128k": Workload("llama3_8b_128k", 32, 1, 8, 128, 8192, 4, 0.5, torch.bfloat16, 131072,
                               rope_base=500000.0, n_q_heads=32),
    "decode_b8_256k": Workload("decode_b8_256k", 32, 8, 32, 128, 4096, 4, 0.5, torch.bfloat16, 262144),
}


class AR1Stream:
    """Stationary AR(1) stream over the token axis for a tensor of shape [*prefix, T, d]."""

    BLOCK = 64

    def __init__(self, prefix, d, rho, seed, device):
        self.prefix, self.d, self.rho = tuple(prefix), d, rho
        self.device = torch.device(device)
        self.gen = torch.Generator(device=self.device)
        self.gen.manual_seed(seed)
        self.state = None
        i = torch.arange(self.BLOCK, device=self.device, dtype=torch.float64)
        diff = i[:, None] - i[None, :]
        self.T = torch.where(diff >= 0, rho ** diff.clamp(min=0), torch.zeros_like(diff)).float()
        self.pw = (rho ** (i + 1)).float()

    def next(self, T: int) -> torch.Tensor:
        e = torch.randn(*self.prefix, T, self.d, generator=self.gen, device=self.device, dtype=torch.float32)
        if self.state is None:
            e[..., 0, :] /= math.sqrt(1.0 - self.rho ** 2)
            self.state = torch.zeros(*self.prefix, self.d, device=self.device)
        out = torch.empty_like(e)
        for t0 in range(0, T, self.BLOCK):
            b = min(self.BLOCK, T - t0)
            blk = torch.matmul(self.T[:b, :b], e[..., t0:t0 + b, :])
            blk += self.pw[:b, None] * self.state[..., None, :]
            out[..., t0:t0 + b, :] = blk
            self.state = blk[..., b - 1, :].clone()
        return out


def rope_rotate(x: torch.Tensor, pos0: int, base: float) -> torch.Tensor:
    """Rotate channel pairs (i, i + d/2) of x[..., T, d] by angle (pos0 + t) * base**(-2i/d)."""
    T, d = x.shape[-2], x.shape[-1]
    half = d // 2
    i = torch.arange(half, device=x.device, dtype=torch.float64)
    theta = base ** (-2.0 * i / d)
    p = torch.arange(pos0, pos0 + T, device=x.device, dtype=torch.float64)
    ang = p[:, None] * theta[None, :]
    c, s = torch.cos(ang).float(), torch.sin(ang).float()
    x1, x2 = x[..., :half], x[..., half:]
    return torch.cat([x1 * c - x2 * s, x1 * s + x2 * c], dim=-1)


def outlier_scale(prefix, d, seed, device, n_outlier=4, factor=8.0) -> torch.Tensor:
    """Per-head channel scale [*prefix, 1, d]: `n_outlier` seeded channels are multiplied by `factor`."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed ^ 0x5EED)
    n = 1
    for p in prefix:
        n *= p
    idx = torch.stack([torch.randperm(d, generator=g)[:n_outlier] for _ in range(n)])
    sc = torch.ones(n, d)
    sc.scatter_(1, idx, factor)
    return sc.reshape(*prefix, 1, d).to(device)


class KVSource:
    """Stream of synthetic K and V chunks for one workload: next(T) -> (K, V) [L, B, H, T, d]."""

    def __init__(self, wl: Workload, seed: int = 0, device="cpu", layer_chunk: int = 8):
        self.wl, self.device, self.pos = wl, torch.device(device), 0
        self.layer_chunk = max(1, min(layer_chunk, wl.n_layers))
        self.groups = []
        for l0 in range(0, wl.n_layers, self.layer_chunk):
            nl = min(self.layer_chunk, wl.n_layers - l0)
            prefix = (nl, wl.batch, wl.n_heads)
            self.groups.append(dict(
                l0=l0, nl=nl,
                k=AR1Stream(prefix, wl.head_dim, wl.rho_k, seed * 1000003 + 2 * l0 + 1, self.device),
                v=AR1Stream(prefix, wl.head_dim, wl.rho_v, seed * 1000003 + 2 * l0 + 2, self.device),
                sc=None if wl.name == "tiny" else outlier_scale(prefix, wl.head_dim, seed * 7919 + l0, self.device),
                noise=torch.Generator(device=self.device).manual_seed(seed * 31 + l0 + 12345),
            ))

    def fill(self, k_out: torch.Tensor, v_out: torch.Tensor, row0: int, T: int) -> None:
        """Write the next T tokens into k_out/v_out[:, :, :, row0:row0+T, :] (layer group by layer group)."""
        wl = self.wl
        for g in self.groups:
            sl = slice(g["l0"], g["l0"] + g["nl"])
            k = g["k"].next(T)
            v = g["v"].next(T)
            if wl.name == "tiny":
                k = k + 0.1 * torch.randn(k.shape, generator=g["noise"], device=self.device)
                v = v + 0.1 * torch.randn(v.shape, generator=g["noise"], device=self.device)
            else:
                k = rope_rotate(k, self.pos, wl.rope_base) * g["sc"]
            k_out[sl, :, :, row0:row0 + T, :] = k.to(k_out.dtype)
            v_out[sl, :, :, row0:row0 + T, :] = v.to(v_out.dtype)
        self.pos += T


def queries(wl: Workload, seed: int, device, scale: float = 0.5) -> torch.Tensor:
    """Seeded decode queries [L, B, Hq, d] ~ N(0, scale^2) in the workload's dtype (un-rotated)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed * 2654435761 % (1 << 31) + 17)
    q = torch.randn(wl.n_layers, wl.batch, wl.q_heads, wl.head_dim, generator=g) * scale
    return q.to(wl.dtype).to(device)


def empty_cache(wl: Workload, device, capacity: int | None = None):
    cap = wl.window if capacity is None else capacity
    shape = (wl.n_layers, wl.batch, wl.n_heads, cap, wl.head_dim)
    return (torch.empty(shape, dtype=wl.dtype, device=device), torch.empty(shape, dtype=wl.dtype, device=device))


def small(wl: Workload, **kw) -> Workload:
    """A reduced copy of a workload (same generator, fewer layers/heads/tokens) for parity tests."""
    d = dict(wl.__dict__)
    d.update(kw)
    return Workload(**d)
