"""Trigger schedule around freqkv_compress (Sec. 3.4): a bounded KV cache that compresses itself, and the
attention calls over it (chunk-wise for prefill, one token for decode; rotary embedding at read time).

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
                 dtype=torch.bfloat16, device="cuda", capacity=None, flags=0, stream=None,
                 n_q_heads=None, rope_base=10000.0):
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
        self.n_q_heads = n_heads if n_q_heads is None else n_q_heads
        self.rope_base = rope_base
        need = max(p.workspace_bytes, 256)
        rc, ap = fk.attend_plan(self.layout, self.n_q_heads, n_heads, head_dim, self.capacity, check=False)
        if rc == fk.OK:
            need = max(need, ap.workspace_bytes)
        rc, pp = fk.attend_prefill_plan(self.layout, self.n_q_heads, n_heads, head_dim, self.capacity, self.capacity,
                                        check=False)
        self.can_prefill = rc == fk.OK
        if self.can_prefill:
            need = max(need, pp.workspace_bytes)
        self.workspace = torch.empty(need, dtype=torch.uint8, device=device)
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

    # ---- attention over [sinks | compressed rows | tokens since], positions = rows of the cache ----------

    def attend_decode(self, q: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
        """q [L, B, Hq, d]: the query of the token appended last (it sits in row cur_len - 1)."""
        out = torch.empty_like(q) if out is None else out
        fk.attend_decode(q, self.k, self.v, out, None, self.layout, self.n_q_heads, self.n_heads, self.head_dim,
                         self.cur_len, -1, self.rope_base, self.stream)
        return out

    def attend_prefill(self, q: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
        """q [L, B, Hq, T, d]: the queries of the T tokens appended last (rows cur_len - T .. cur_len - 1)."""
        out = torch.empty_like(q) if out is None else out
        fk.attend_prefill(q, self.k, self.v, out, None, self.layout, self.n_q_heads, self.n_heads, self.head_dim,
                          self.cur_len, q.shape[3], self.rope_base, self.stream)
        return out

    def prefill(self, k_new: torch.Tensor, v_new: torch.Tensor, q_new: torch.Tensor) -> torch.Tensor:
        """Chunk-wise prefill of Sec. 3.4: K/V/q of T new tokens ([L, B, H|Hq, T, d]); the tokens go into the
        cache in pieces that fit (a trigger whenever it is full and tokens remain) and every piece attends to
        the cache as it stands then.  Returns the attention outputs [L, B, Hq, T, d]."""
        T, t0 = k_new.shape[3], 0
        out = torch.empty_like(q_new)
        while t0 < T:
            if self.cur_len >= self.window:
                self.compress()
            take = min(T - t0, self.window - self.cur_len)
            self.k[:, :, :, self.cur_len:self.cur_len + take] = k_new[:, :, :, t0:t0 + take]
            self.v[:, :, :, self.cur_len:self.cur_len + take] = v_new[:, :, :, t0:t0 + take]
            self.cur_len += take
            out[:, :, :, t0:t0 + take] = self.attend_prefill(q_new[:, :, :, t0:t0 + take].contiguous())
            t0 += take
        return out
