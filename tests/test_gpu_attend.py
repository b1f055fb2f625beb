"""GPU parity of freqkv_attend_decode (HIP, through the C ABI) against the fp64 attention oracle.

The oracle sees exactly the bits the GPU sees.  Tolerances (derived in the design notes):
  bf16: the output is one rounding of an fp32 result, so |err| <= half a bf16 ulp of the reference plus
        the fp32 error below;
  fp32: |err| <= 2e-6 * max|v| (fp32 scores of a few units, hardware exp2, a cos/sin recurrence of at
        most 64 steps between exact seeds).
"""
import math

import numpy as np
import pytest
import torch

import paper_2505_00570_amd as fk
from paper_2505_00570_amd import binding, synth
from oracle import attend_oracle as att
from oracle import freqkv_oracle as orc

from _util import bf16_ulp, f64

pytestmark = pytest.mark.gpu
DEV = "cuda"
TOL_ATT_F32 = 2e-6


def _say(msg):
    print(msg, flush=True)


def _wl(d=128, hkv=2, hq=8, layers=1, batch=1, cap=512, dtype=torch.bfloat16, base=10000.0):
    return synth.small(synth.WORKLOADS["llama3_8b_128k"], n_layers=layers, batch=batch, n_heads=hkv, n_q_heads=hq,
                       head_dim=d, window=cap, dtype=dtype, rope_base=base, total_tokens=cap)


def _mk(wl, cur_len, seed=0, cap=None):
    cap = cap or wl.window
    k, v = synth.empty_cache(wl, DEV, cap)
    k.fill_(float("nan"))          # rows at and beyond cur_len must never influence the result
    v.fill_(float("nan"))
    synth.KVSource(wl, seed, DEV).fill(k, v, 0, cur_len)
    q = synth.queries(wl, seed, DEV)
    return q, k, v


def _run(q, k, v, wl, cur_len, q_pos=-1, base=None, want_lse=True, layout=None, kk=None, vv=None):
    L = layout or binding.layout_for(k)
    _, p = fk.attend_plan(L, wl.q_heads, wl.n_heads, wl.head_dim, cur_len)
    ws = torch.empty(max(p.workspace_bytes, 256), dtype=torch.uint8, device=DEV)
    L.workspace, L.workspace_bytes = ws.data_ptr(), p.workspace_bytes
    out = torch.full_like(q, float("nan"))
    lse = torch.full(q.shape[:3], float("nan"), dtype=torch.float32, device=DEV) if want_lse else None
    fk.attend_decode(q, k if kk is None else kk, v if vv is None else vv, out, lse, L, wl.q_heads, wl.n_heads,
                     wl.head_dim, cur_len, q_pos, wl.rope_base if base is None else base)
    torch.cuda.synchronize()
    return out, lse, p


def _check(q, k, v, out, lse, wl, cur_len, q_pos=None, base=None, heads=None):
    base = wl.rope_base if base is None else base
    worst = 0.0
    qh, kh, vh, oh = q.cpu(), k.cpu(), v.cpu(), out.cpu()
    lh = lse.cpu() if lse is not None else None
    for l in range(wl.n_layers):
        for b in range(wl.batch):
            ref, rlse = att.attend_decode(f64(qh[l, b]), f64(kh[l, b, :, :cur_len]), f64(vh[l, b, :, :cur_len]),
                                          cur_len, q_pos, base if base > 0 else 10000.0, rope=base > 0)
            got = f64(oh[l, b])
            assert not np.isnan(got).any(), (l, b)
            vmax = float(np.abs(f64(vh[l, b, :, :cur_len])).max())
            err = np.abs(got - ref)
            if wl.dtype == torch.bfloat16:
                bound = 0.5 * bf16_ulp(ref) * 1.001 + TOL_ATT_F32 * vmax
            else:
                bound = np.full_like(ref, TOL_ATT_F32 * vmax)
            assert (err <= bound).all(), (l, b, float(err.max()), float((err / bound).max()))
            worst = max(worst, float((err / bound).max()))
            if lh is not None:
                assert np.max(np.abs(f64(lh[l, b]) - rlse)) <= 2e-5 * (1.0 + np.abs(rlse).max()), (l, b)
    return worst


@pytest.mark.parametrize("cur_len", [1, 2, 7, 31, 32, 33, 64, 65, 200, 511, 512])
def test_bf16_d128_gqa4_lengths(cur_len):
    wl = _wl()
    _say(f"attend bf16 d128 G4 cur_len={cur_len}")
    q, k, v = _mk(wl, cur_len, seed=cur_len)
    out, lse, p = _run(q, k, v, wl, cur_len)
    w = _check(q, k, v, out, lse, wl, cur_len)
    _say(f"  n_split={p.n_split} chunk={p.chunk_rows} worst err/bound={w:.3f}")


@pytest.mark.parametrize("d,hkv,hq", [(64, 2, 2), (64, 1, 4), (128, 4, 4), (128, 2, 4), (128, 1, 8), (128, 1, 3),
                                      (128, 2, 12), (256, 2, 4), (256, 1, 1)])
def test_bf16_head_shapes(d, hkv, hq):
    wl = _wl(d=d, hkv=hkv, hq=hq, cap=700, layers=2, batch=2)
    cur_len = 611
    _say(f"attend bf16 d={d} hkv={hkv} hq={hq}")
    q, k, v = _mk(wl, cur_len, seed=d + hq)
    out, lse, p = _run(q, k, v, wl, cur_len)
    assert p.heads_together in (1, 2, 4) and (hq // hkv) % p.heads_together == 0
    w = _check(q, k, v, out, lse, wl, cur_len)
    _say(f"  GT={p.heads_together} n_split={p.n_split} worst err/bound={w:.3f}")


@pytest.mark.parametrize("d,cur_len", [(64, 300), (128, 1000), (256, 129)])
def test_fp32(d, cur_len):
    wl = _wl(d=d, hkv=2, hq=4, cap=1024, dtype=torch.float32)
    _say(f"attend fp32 d={d} cur_len={cur_len}")
    q, k, v = _mk(wl, cur_len, seed=3)
    out, lse, p = _run(q, k, v, wl, cur_len)
    w = _check(q, k, v, out, lse, wl, cur_len)
    _say(f"  worst err/bound={w:.3f}")


def test_long_cache_many_chunks():
    """The LLaMA-3 window (8192 rows, base 500000) on two layers: several chunks per KV head."""
    wl = _wl(hkv=8, hq=32, layers=2, cap=8192, base=500000.0)
    q, k, v = _mk(wl, 8192, seed=5)
    out, lse, p = _run(q, k, v, wl, 8192)
    assert p.n_split > 1
    w = _check(q, k, v, out, lse, wl, 8192)
    _say(f"attend 8192 rows: n_split={p.n_split} chunk={p.chunk_rows} worst err/bound={w:.3f}")


def test_without_rotary_and_explicit_query_position():
    wl = _wl(cap=400)
    q, k, v = _mk(wl, 333, seed=9)
    out, lse, _ = _run(q, k, v, wl, 333, base=0.0)
    _check(q, k, v, out, lse, wl, 333, base=0.0)
    out2, lse2, _ = _run(q, k, v, wl, 333, q_pos=100)
    _check(q, k, v, out2, lse2, wl, 333, q_pos=100)
    out3, _, _ = _run(q, k, v, wl, 333, q_pos=332, want_lse=False)
    out4, _, _ = _run(q, k, v, wl, 333)
    assert torch.equal(out3, out4)                    # -1 means cur_len - 1
    assert not torch.equal(out2, out4)


def test_token_major_cache_and_pointer_table():
    import ctypes as C
    wl = _wl(hkv=2, hq=4, layers=3, batch=2, cap=256)
    cur = 201
    q, k, v = _mk(wl, cur, seed=11)
    ref_out, ref_lse, _ = _run(q, k, v, wl, cur)
    # token-major storage [layer, batch, token, head, dim] viewed as [layer, batch, head, token, dim]
    kt = k.permute(0, 1, 3, 2, 4).contiguous().permute(0, 1, 3, 2, 4)
    vt = v.permute(0, 1, 3, 2, 4).contiguous().permute(0, 1, 3, 2, 4)
    assert kt.stride(3) == wl.n_heads * wl.head_dim
    out, lse, _ = _run(q, kt, vt, wl, cur)
    assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse)
    # per-layer allocations behind a host pointer table
    ks = [k[l].clone() for l in range(wl.n_layers)]
    vs = [v[l].clone() for l in range(wl.n_layers)]
    L = binding.layout_for(k)
    L.pointer_table = 1
    kp = (C.c_void_p * wl.n_layers)(*[t.data_ptr() for t in ks])
    vp = (C.c_void_p * wl.n_layers)(*[t.data_ptr() for t in vs])
    out, lse, _ = _run(q, k, v, wl, cur, layout=L, kk=kp, vv=vp)
    assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse)


def test_more_layers_than_one_pass_holds():
    wl = _wl(d=64, hkv=1, hq=2, layers=100, cap=64)
    q, k, v = _mk(wl, 50, seed=13)
    out, lse, _ = _run(q, k, v, wl, 50)
    _check(q, k, v, out, lse, wl, 50)


def test_errors_leave_output_untouched():
    wl = _wl(cap=128)
    q, k, v = _mk(wl, 100, seed=1)
    L = binding.layout_for(k)
    _, p = fk.attend_plan(L, wl.q_heads, wl.n_heads, wl.head_dim, 100)
    ws = torch.empty(p.workspace_bytes, dtype=torch.uint8, device=DEV)
    out = torch.full_like(q, 5.0)
    args = dict(stream=None, check=False)
    # no workspace
    assert fk.attend_decode(q, k, v, out, None, L, wl.q_heads, wl.n_heads, wl.head_dim, 100, **args) == -3
    L.workspace, L.workspace_bytes = ws.data_ptr(), p.workspace_bytes - 1
    assert fk.attend_decode(q, k, v, out, None, L, wl.q_heads, wl.n_heads, wl.head_dim, 100, **args) == -3
    L.workspace_bytes = p.workspace_bytes
    assert fk.attend_decode(q, k, v, out, None, L, wl.q_heads, wl.n_heads, wl.head_dim, 0, **args) == -1
    assert fk.attend_decode(q, k, v, out, None, L, wl.q_heads, wl.n_heads, wl.head_dim, 129, **args) == -1
    assert fk.attend_decode(q, k, v, out, None, L, 7, wl.n_heads, wl.head_dim, 100, **args) == -1
    assert fk.attend_decode(q, k, v, out, None, L, wl.q_heads, wl.n_heads, 96, 100, **args) == -2
    assert fk.attend_decode(q, k, v, out, None, L, wl.q_heads, wl.n_heads, wl.head_dim, 100, q_pos=-2, **args) == -1
    assert fk.attend_decode(q, k, v, out, None, L, wl.q_heads, wl.n_heads, wl.head_dim, 100,
                            rope_base=float("nan"), **args) == -1
    assert fk.attend_decode(None, k, v, out, None, L, wl.q_heads, wl.n_heads, wl.head_dim, 100, **args) == -1
    torch.cuda.synchronize()
    assert bool((out == 5.0).all())


def test_compress_then_attend():
    """The step after a trigger: attention over [sinks | compressed rows | tail] of the cache the library
    itself compacted, checked against the oracle on those same bits, and against the all-oracle path."""
    wl = synth.small(synth.WORKLOADS["llama3_8b_128k"], n_layers=1, n_heads=2, n_q_heads=8, window=512)
    cur = 520
    k, v = synth.empty_cache(wl, DEV, 600)
    k.fill_(float("nan")); v.fill_(float("nan"))
    synth.KVSource(wl, 21, DEV).fill(k, v, 0, cur)
    k0, v0 = k.clone(), v.clone()
    q = synth.queries(wl, 21, DEV)
    L = binding.layout_for(k)
    _, p = fk.plan(L, wl.n_heads, wl.head_dim, cur, wl.window, wl.n_sink, wl.retain_ratio)
    ws = torch.empty(p.workspace_bytes, dtype=torch.uint8, device=DEV)
    L.workspace, L.workspace_bytes = ws.data_ptr(), p.workspace_bytes
    fk.compress(k, v, L, wl.n_heads, wl.head_dim, cur, wl.window, wl.n_sink, wl.retain_ratio)
    torch.cuda.synchronize()
    new_len = p.new_len
    assert new_len == wl.n_sink + p.retained_len + (cur - wl.window)
    k[:, :, :, new_len:] = float("nan")       # whatever lies beyond the compacted cache must not matter
    v[:, :, :, new_len:] = float("nan")
    out, lse, _ = _run(q, k, v, wl, new_len)
    _check(q, k, v, out, lse, wl, new_len)
    # all-oracle path: fp64 compression of the original rows, then fp64 attention; the difference is the
    # bf16 rounding of the compressed rows carried through the softmax
    worst = 0.0
    for b in range(wl.batch):
        kc = np.stack([orc.compress_head(f64(k0[0, b, h, :cur].cpu()), cur, wl.window, wl.n_sink, wl.retain_ratio)
                       for h in range(wl.n_heads)])
        vc = np.stack([orc.compress_head(f64(v0[0, b, h, :cur].cpu()), cur, wl.window, wl.n_sink, wl.retain_ratio)
                       for h in range(wl.n_heads)])
        ref, _ = att.attend_decode(f64(q[0, b].cpu()), kc, vc, new_len, None, wl.rope_base)
        got = f64(out[0, b].cpu())
        rms = math.sqrt(float((ref ** 2).mean()))
        worst = max(worst, float(np.abs(got - ref).max()) / rms)
    _say(f"compress->attend vs all-fp64 path: max err / rms = {worst:.3e}")
    assert worst < 5e-2


# ---------------------------------------------------------------- batches of unequal cache lengths

def _run_ragged(q, k, v, wl, lens, max_len=None):
    L = binding.layout_for(k)
    max_len = max_len or max(lens)
    _, p = fk.attend_plan(L, wl.q_heads, wl.n_heads, wl.head_dim, max_len)
    ws = torch.empty(max(p.workspace_bytes, 256), dtype=torch.uint8, device=DEV)
    L.workspace, L.workspace_bytes = ws.data_ptr(), p.workspace_bytes
    out = torch.full_like(q, float("nan"))
    lse = torch.full(q.shape[:3], float("nan"), dtype=torch.float32, device=DEV)
    cl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    fk.attend_decode_ragged(q, k, v, out, lse, L, wl.q_heads, wl.n_heads, wl.head_dim, cl, max_len, wl.rope_base)
    torch.cuda.synchronize()
    return out, lse, p


@pytest.mark.parametrize("lens", [[1, 37, 300, 512], [512, 512, 512, 512], [64, 1, 2, 33], [500, 17, 499, 256]])
def test_ragged_batch(lens):
    wl = _wl(hkv=2, hq=8, layers=2, batch=4, cap=512)
    _say(f"attend ragged lens={lens}")
    k, v = synth.empty_cache(wl, DEV, 512)
    synth.KVSource(wl, 31, DEV).fill(k, v, 0, 512)
    for b, n in enumerate(lens):                   # rows a sequence does not hold must not matter
        k[:, b, :, n:] = float("nan")
        v[:, b, :, n:] = float("nan")
    q = synth.queries(wl, 31, DEV)
    out, lse, p = _run_ragged(q, k, v, wl, lens)
    for b, n in enumerate(lens):
        sub = synth.small(wl, batch=1)
        _check(q[:, b:b + 1], k[:, b:b + 1], v[:, b:b + 1], out[:, b:b + 1], lse[:, b:b + 1], sub, n)
    if len(set(lens)) == 1:                        # equal lengths: the same bits as the uniform entry point
        k2, v2 = k.clone(), v.clone()
        ref, rlse, _ = _run(q, k2, v2, wl, lens[0])
        assert torch.equal(ref, out) and torch.equal(rlse, lse)


def test_ragged_long_and_short_with_many_chunks():
    wl = _wl(hkv=2, hq=8, layers=1, batch=3, cap=4096, base=500000.0)
    lens = [4096, 5, 1700]
    k, v = synth.empty_cache(wl, DEV, 4096)
    synth.KVSource(wl, 41, DEV).fill(k, v, 0, 4096)
    for b, n in enumerate(lens):
        k[:, b, :, n:] = float("nan")
        v[:, b, :, n:] = float("nan")
    q = synth.queries(wl, 41, DEV)
    out, lse, p = _run_ragged(q, k, v, wl, lens)
    assert p.n_split > 1                           # the short sequences leave whole chunks empty
    for b, n in enumerate(lens):
        sub = synth.small(wl, batch=1)
        _check(q[:, b:b + 1], k[:, b:b + 1], v[:, b:b + 1], out[:, b:b + 1], lse[:, b:b + 1], sub, n)


def test_ragged_lengths_are_clamped_on_the_device():
    """Values outside [1, max_cur_len] in the device array cannot make the kernel leave the cache."""
    wl = _wl(hkv=1, hq=4, layers=1, batch=3, cap=128)
    k, v = synth.empty_cache(wl, DEV, 128)
    synth.KVSource(wl, 43, DEV).fill(k, v, 0, 128)
    q = synth.queries(wl, 43, DEV)
    out, lse, _ = _run_ragged(q, k, v, wl, [0, -7, 10 ** 6], max_len=100)
    ref, rlse, _ = _run_ragged(q, k, v, wl, [1, 1, 100], max_len=100)
    assert torch.equal(out, ref) and torch.equal(lse, rlse)


def test_ragged_errors():
    wl = _wl(hkv=1, hq=4, layers=1, batch=2, cap=128)
    q, k, v = _mk(wl, 128, seed=2)
    L = binding.layout_for(k)
    _, p = fk.attend_plan(L, wl.q_heads, wl.n_heads, wl.head_dim, 128)
    ws = torch.empty(p.workspace_bytes, dtype=torch.uint8, device=DEV)
    L.workspace, L.workspace_bytes = ws.data_ptr(), p.workspace_bytes
    out = torch.full_like(q, 5.0)
    cl = torch.tensor([3, 4], dtype=torch.int32, device=DEV)
    f = fk.attend_decode_ragged
    assert f(q, k, v, out, None, L, wl.q_heads, wl.n_heads, wl.head_dim, None, 128, check=False) == -1
    assert f(q, k, v, out, None, L, wl.q_heads, wl.n_heads, wl.head_dim, cl, 0, check=False) == -1
    assert f(q, k, v, out, None, L, wl.q_heads, wl.n_heads, wl.head_dim, cl, 129, check=False) == -1
    torch.cuda.synchronize()
    assert bool((out == 5.0).all())


# ---------------------------------------------------------------- the benchmark's full sizes, sampled

def _sampled_full(wl_name, n_pick, seed):
    """All layers of a benchmark workload in one call (the launch configuration bench.py times); the oracle
    checks a seeded sample of (layer, batch) slices that always holds the first and the last one."""
    wl = synth.WORKLOADS[wl_name]
    cur = wl.window
    k, v = synth.empty_cache(wl, DEV)
    synth.KVSource(wl, seed, DEV).fill(k, v, 0, cur)
    q = synth.queries(wl, seed, DEV)
    out, lse, p = _run(q, k, v, wl, cur)
    assert not torch.isnan(out.float()).any()
    rng = np.random.default_rng(seed)
    picks = {(0, 0), (wl.n_layers - 1, wl.batch - 1)}
    while len(picks) < n_pick:
        picks.add((int(rng.integers(wl.n_layers)), int(rng.integers(wl.batch))))
    worst = 0.0
    for l, b in sorted(picks):
        kk, vv = f64(k[l, b].cpu()), f64(v[l, b].cpu())
        ref, rlse = att.attend_decode(f64(q[l, b].cpu()), kk, vv, cur, None, wl.rope_base)
        vmax = float(np.abs(vv).max())
        err = np.abs(f64(out[l, b].cpu()) - ref)
        bound = 0.5 * bf16_ulp(ref) * 1.001 + TOL_ATT_F32 * vmax
        assert (err <= bound).all(), (l, b, float((err / bound).max()))
        worst = max(worst, float((err / bound).max()))
        assert np.max(np.abs(f64(lse[l, b].cpu()) - rlse)) <= 2e-5 * (1.0 + np.abs(rlse).max())
    _say(f"attend {wl_name}: n_split={p.n_split} GT={p.heads_together}, {len(picks)} slices, worst err/bound={worst:.3f}")


def test_full_llama3_8b_128k():
    _sampled_full("llama3_8b_128k", 4, 1)


def test_full_llama2_7b_32k():
    _sampled_full("llama2_7b_32k", 3, 2)


def test_full_decode_b8_256k():
    _sampled_full("decode_b8_256k", 4, 3)
