"""Trigger schedule around freqkv_compress (Sec. 3.4): a bounded KV cache that compresses itself.

Thin host logic only: it owns the K/V tensors, the workspace and `cur_len`, asks freqkv_plan for
the lengths, and calls freqkv_compress when the cache is full and more tokens arrive (the lazy
trigger that yields the paper's compression counts: none at 4K, 3 at 8K, ... 127 at 256K for a
4096-token window).  All arithmetic on cache contents happens inside libfreqkv.
"""
from __future__ import annotations

import torch

from . import binding as fk


class CompressedKVCache:
    def __init__(self, n_layers, batch, n_heads, head_dim, window, n_sink=4, retain_ratio=0.5,
                 dtype=torch.bfloat16, device="cuda", capacity=None, flags=0, stream=None):
        self.window, self.n_sink, self.retain_ratio = window, n_sink, retain_ratio
        self.n_heads, self.head_dim = n_heads, head_dim
        self.capacity = window if capacity is None else capacity
        shape = (n_layers, batch, n_heads, self.capacity, head_dim)
        self.k = torch.empty(shape, dtype=dtype, device=device)
        self.v = torch.empty(shape, dtype=dtype, device=device)
        self.cur_len = 0
        self.triggers = 0
        self.stream = stream
        self.layout = fk.layout_for(self.k, flags=flags)
        _, p = fk.plan(self.layout, n_heads, head_dim, window, window, n_sink, retain_ratio)
        self.plan = p
        self.workspace = torch.empty(max(p.workspace_bytes, 256), dtype=torch.uint8, device=device)
        self.layout.workspace = self.workspace.data_ptr()
        self.layout.workspace_bytes = self.workspace.numel()

    @property
    def free_after_trigger(self) -> int:
        return self.window - self.n_sink - self.plan.retained_len

    def compress(self) -> int:
        """One trigger (if the cache is full); returns the library status."""
        rc = fk.compress(self.k, self.v, self.layout, self.n_heads, self.head_dim, self.cur_len,
                         self.window, self.n_sink, self.retain_ratio, self.stream)
        if rc == fk.OK and self.cur_len >= self.window:
            _, p = fk.plan(self.layout, self.n_heads, self.head_dim, self.cur_len, self.window,
                           self.n_sink, self.retain_ratio)
            self.cur_len = p.new_len
            self.triggers += 1
        return rc

    def room(self) -> int:
        return self.window - self.cur_len

    def append(self, k_new: torch.Tensor, v_new: torch.Tensor) -> None:
        """Append [L, B, H, T, d] tokens, compressing whenever the cache is full and tokens remain."""
        T, t0 = k_new.shape[3], 0
        while t0 < T:
            if self.cur_len >= self.window:
                self.compress()
            take = min(T - t0, self.window - self.cur_len)
            self.k[:, :, :, self.cur_len:self.cur_len + take] = k_new[:, :, :, t0:t0 + take]
            self.v[:, :, :, self.cur_len:self.cur_len + take] = v_new[:, :, :, t0:t0 + take]
            self.cur_len += take
            t0 += take
