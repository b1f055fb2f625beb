"""The pieces together on a small cache: chunk-wise prefill with triggers in between, then token-by-token
decoding, through paper_2505_00570_amd.cache.CompressedKVCache.  Every attention output is compared with the
fp64 oracle evaluated on the very cache bits the GPU holds at that moment (so each comparison isolates one
attention call; the compression itself is checked in test_gpu_parity.py), and the schedule is compared with
the oracle's integer rules."""
import numpy as np
import pytest
import torch

from paper_2505_00570_amd import synth
from paper_2505_00570_amd.cache import CompressedKVCache
from oracle import attend_oracle as att
from oracle import freqkv_oracle as orc

from _util import bf16_ulp, f64

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _check(out, ref, vmax, tol):
    err = np.abs(f64(out) - ref)
    over = np.maximum(err - 0.5 * bf16_ulp(ref) * 1.001, 0.0) / vmax
    assert float(over.max()) <= tol, float(over.max())
    return float(over.max())


def test_prefill_then_decode_session():
    wl = synth.small(synth.WORKLOADS["llama3_8b_128k"], n_layers=2, batch=1, n_heads=2, n_q_heads=4, window=132,
                     total_tokens=700)
    cache = CompressedKVCache(wl.n_layers, wl.batch, wl.n_heads, wl.head_dim, wl.window, wl.n_sink, wl.retain_ratio,
                              n_q_heads=wl.q_heads, rope_base=wl.rope_base, device=DEV)
    assert cache.can_prefill
    src = synth.KVSource(wl, 3, DEV)
    g = torch.Generator(device="cpu").manual_seed(5)
    total, done, worst = 600, 0, 0.0
    lc = orc.retained_len(wl.window - wl.n_sink, wl.retain_ratio)
    while done < total:                                # prompts arrive in pieces of 50 tokens
        T = min(50, total - done)
        kn, vn = synth.empty_cache(synth.small(wl, window=T), DEV, T)
        src.fill(kn, vn, 0, T)
        qn = (torch.randn(wl.n_layers, 1, wl.q_heads, T, wl.head_dim, generator=g) * 0.5).to(torch.bfloat16).to(DEV)
        # replay the cache driver's own splitting so that each attention call can be checked on its own
        t0 = 0
        while t0 < T:
            if cache.cur_len >= cache.window:
                cache.compress()
                assert cache.cur_len == wl.n_sink + lc
            take = min(T - t0, cache.window - cache.cur_len)
            cache.k[:, :, :, cache.cur_len:cache.cur_len + take] = kn[:, :, :, t0:t0 + take]
            cache.v[:, :, :, cache.cur_len:cache.cur_len + take] = vn[:, :, :, t0:t0 + take]
            cache.cur_len += take
            q = qn[:, :, :, t0:t0 + take].contiguous()
            out = cache.attend_prefill(q)
            torch.cuda.synchronize()
            for l in range(wl.n_layers):
                kk, vv = f64(cache.k[l, 0, :, :cache.cur_len].cpu()), f64(cache.v[l, 0, :, :cache.cur_len].cpu())
                ref, _ = att.attend_prefill(f64(q[l, 0].cpu()), kk, vv, cache.cur_len, wl.rope_base)
                worst = max(worst, _check(out[l, 0].cpu(), ref, float(np.abs(vv).max()), 2e-3))
            t0 += take
        done += T
    assert cache.triggers == orc.trigger_count(total, wl.window, wl.n_sink, wl.retain_ratio)
    # decoding: one token at a time, a trigger whenever the cache is full
    for step in range(40):
        kn, vn = synth.empty_cache(synth.small(wl, window=1), DEV, 1)
        src.fill(kn, vn, 0, 1)
        cache.append(kn, vn)
        q = (torch.randn(wl.n_layers, 1, wl.q_heads, wl.head_dim, generator=g) * 0.5).to(torch.bfloat16).to(DEV)
        out = cache.attend_decode(q)
        torch.cuda.synchronize()
        for l in range(wl.n_layers):
            kk, vv = f64(cache.k[l, 0, :, :cache.cur_len].cpu()), f64(cache.v[l, 0, :, :cache.cur_len].cpu())
            ref, _ = att.attend_decode(f64(q[l, 0].cpu()), kk, vv, cache.cur_len, None, wl.rope_base)
            _check(out[l, 0].cpu(), ref, float(np.abs(vv).max()), 2e-6)
    assert cache.triggers == orc.trigger_count(total + 40, wl.window, wl.n_sink, wl.retain_ratio)
    print(f"session: {cache.triggers} triggers, worst prefill excess / max|V| = {worst:.2e}", flush=True)


def test_prefill_method_equals_manual_pieces():
    wl = synth.small(synth.WORKLOADS["llama3_8b_128k"], n_layers=1, batch=1, n_heads=1, n_q_heads=4, window=100)
    mk = lambda: CompressedKVCache(1, 1, 1, 128, 100, 4, 0.5, n_q_heads=4, rope_base=wl.rope_base, device=DEV)
    a, b = mk(), mk()
    src = synth.KVSource(wl, 9, DEV)
    kn, vn = synth.empty_cache(synth.small(wl, window=260), DEV, 260)
    src.fill(kn, vn, 0, 260)
    qn = (torch.randn(1, 1, 4, 260, 128, generator=torch.Generator().manual_seed(2)) * 0.5).to(torch.bfloat16).to(DEV)
    out = a.prefill(kn, vn, qn)
    # the same by hand: 100 tokens fill the window, then pieces of 100 - 4 - 48 = 48 tokens after each trigger
    pieces, t0 = [], 0
    while t0 < 260:
        if b.cur_len >= b.window:
            b.compress()
        take = min(260 - t0, b.window - b.cur_len)
        b.k[:, :, :, b.cur_len:b.cur_len + take] = kn[:, :, :, t0:t0 + take]
        b.v[:, :, :, b.cur_len:b.cur_len + take] = vn[:, :, :, t0:t0 + take]
        b.cur_len += take
        pieces.append(b.attend_prefill(qn[:, :, :, t0:t0 + take].contiguous()))
        t0 += take
    torch.cuda.synchronize()
    assert [p.shape[3] for p in pieces] == [100, 48, 48, 48, 16]
    assert torch.equal(out, torch.cat(pieces, dim=3))
    assert a.triggers == b.triggers == 4 and a.cur_len == b.cur_len
