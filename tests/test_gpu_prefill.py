"""GPU parity of freqkv_attend_prefill (chunk-wise attention on the matrix cores) against the fp64 oracle.

Tolerance: the operands of the matrix cores are fp16 (cache values exactly, rotated keys and scaled rotated
queries rounded to 11 significant bits, softmax weights rounded to 11 bits), everything else fp32, one final
rounding to bf16:  |err| <= half a bf16 ulp of the reference + TOL_PREFILL * max|V|  (derivation in the
design notes; the measured share of TOL_PREFILL is printed by every case).
"""
import math

import numpy as np
import pytest
import torch

import paper_2505_00570_amd as fk
from paper_2505_00570_amd import binding, synth
from oracle import attend_oracle as att

from _util import bf16_ulp, f64

pytestmark = pytest.mark.gpu
DEV = "cuda"
TOL_PREFILL = 2e-3


def _say(msg):
    print(msg, flush=True)


def _wl(hkv=2, hq=8, layers=1, batch=1, cap=512, base=10000.0):
    return synth.small(synth.WORKLOADS["llama3_8b_128k"], n_layers=layers, batch=batch, n_heads=hkv, n_q_heads=hq,
                       head_dim=128, window=cap, rope_base=base, total_tokens=cap)


def _mk(wl, cur_len, q_len, seed=0):
    k, v = synth.empty_cache(wl, DEV, wl.window)
    k.fill_(float("nan"))
    v.fill_(float("nan"))
    synth.KVSource(wl, seed, DEV).fill(k, v, 0, cur_len)
    g = torch.Generator(device="cpu").manual_seed(seed + 1000)
    q = (torch.randn(wl.n_layers, wl.batch, wl.q_heads, q_len, wl.head_dim, generator=g) * 0.5).to(torch.bfloat16).to(DEV)
    return q, k, v


def _run(q, k, v, wl, cur_len, base=None, want_lse=True):
    q_len = q.shape[3]
    L = binding.layout_for(k)
    _, p = fk.attend_prefill_plan(L, wl.q_heads, wl.n_heads, wl.head_dim, cur_len, q_len)
    ws = torch.empty(p.workspace_bytes, dtype=torch.uint8, device=DEV)
    L.workspace, L.workspace_bytes = ws.data_ptr(), p.workspace_bytes
    out = torch.full_like(q, float("nan"))
    lse = torch.full(q.shape[:4], float("nan"), dtype=torch.float32, device=DEV) if want_lse else None
    fk.attend_prefill(q, k, v, out, lse, L, wl.q_heads, wl.n_heads, wl.head_dim, cur_len, q_len,
                      wl.rope_base if base is None else base)
    torch.cuda.synchronize()
    return out, lse, p


def _check(q, k, v, out, lse, wl, cur_len, base=None, rows=None, lse_tol=2e-2):
    """Compare against the oracle; `rows` selects query rows (default: all)."""
    base = wl.rope_base if base is None else base
    q_len = q.shape[3]
    worst = 0.0
    qh, kh, vh, oh = q.cpu(), k.cpu(), v.cpu(), out.cpu()
    lh = lse.cpu() if lse is not None else None
    assert not torch.isnan(oh.float()).any()
    for l in range(wl.n_layers):
        for b in range(wl.batch):
            kk, vv = f64(kh[l, b, :, :cur_len]), f64(vh[l, b, :, :cur_len])
            vmax = float(np.abs(vv).max())
            qq = f64(qh[l, b])
            if rows is None:
                ref, rlse = att.attend_prefill(qq, kk, vv, cur_len, base if base > 0 else 1e4, rope=base > 0)
                got, glse = f64(oh[l, b]), (f64(lh[l, b]) if lh is not None else None)
            else:
                g = wl.q_heads // wl.n_heads
                ref = np.zeros((wl.q_heads, len(rows), wl.head_dim)); rlse = np.zeros((wl.q_heads, len(rows)))
                for h in range(wl.q_heads):
                    for n, i in enumerate(rows):
                        pos = cur_len - q_len + i
                        ref[h, n], rlse[h, n] = att.attend_decode_head(qq[h, i], kk[h // g], vv[h // g], pos + 1, pos,
                                                                       base if base > 0 else 1e4, base > 0)
                got = f64(oh[l, b][:, rows]); glse = f64(lh[l, b][:, rows]) if lh is not None else None
            err = np.abs(got - ref)
            over = np.maximum(err - 0.5 * bf16_ulp(ref) * 1.001, 0.0) / vmax
            worst = max(worst, float(over.max()))
            if glse is not None:
                assert np.max(np.abs(glse - rlse)) <= lse_tol, float(np.max(np.abs(glse - rlse)))
    return worst


@pytest.mark.parametrize("cur_len,q_len", [(1, 1), (31, 31), (32, 5), (33, 33), (64, 64), (65, 1), (100, 37), (200, 200),
                                           (257, 130), (512, 64), (500, 300)])
def test_prefill_lengths(cur_len, q_len):
    wl = _wl()
    _say(f"prefill G4 cur_len={cur_len} q_len={q_len}")
    q, k, v = _mk(wl, cur_len, q_len, seed=cur_len + q_len)
    out, lse, p = _run(q, k, v, wl, cur_len)
    w = _check(q, k, v, out, lse, wl, cur_len)
    _say(f"  worst excess / max|V| = {w:.2e}  ({w / TOL_PREFILL:.2f} of the tolerance)")
    assert w <= TOL_PREFILL


@pytest.mark.parametrize("hkv,hq", [(4, 4), (2, 4), (1, 8), (1, 3), (2, 12), (1, 1)])
def test_prefill_head_groupings(hkv, hq):
    wl = _wl(hkv=hkv, hq=hq, layers=2, batch=2, cap=300)
    cur_len, q_len = 290, 150
    _say(f"prefill hkv={hkv} hq={hq}")
    q, k, v = _mk(wl, cur_len, q_len, seed=hq * 10 + hkv)
    out, lse, _ = _run(q, k, v, wl, cur_len)
    w = _check(q, k, v, out, lse, wl, cur_len)
    _say(f"  worst excess / max|V| = {w:.2e}")
    assert w <= TOL_PREFILL


def test_prefill_unit_count_that_is_not_a_multiple_of_eight():
    """Workgroups are dealt to the KV units in groups of eight units; 11 units = one full group and a remainder."""
    wl = _wl(hkv=11, hq=22, layers=1, batch=1, cap=200)
    cur_len, q_len = 190, 97
    q, k, v = _mk(wl, cur_len, q_len, seed=5)
    out, lse, _ = _run(q, k, v, wl, cur_len)
    w = _check(q, k, v, out, lse, wl, cur_len)
    _say(f"11 KV units: worst excess / max|V| = {w:.2e}")
    assert w <= TOL_PREFILL


def test_prefill_last_query_is_the_decode_case_and_rope_off():
    wl = _wl(cap=400)
    q, k, v = _mk(wl, 333, 70, seed=4)
    out, lse, _ = _run(q, k, v, wl, 333)
    # decode entry point on the last query: same mathematics, fp32 vector path
    L = binding.layout_for(k)
    _, dp = fk.attend_plan(L, wl.q_heads, wl.n_heads, wl.head_dim, 333)
    ws = torch.empty(dp.workspace_bytes, dtype=torch.uint8, device=DEV)
    L.workspace, L.workspace_bytes = ws.data_ptr(), dp.workspace_bytes
    qd = q[:, :, :, -1].contiguous()
    od = torch.empty_like(qd)
    fk.attend_decode(qd, k, v, od, None, L, wl.q_heads, wl.n_heads, wl.head_dim, 333, -1, wl.rope_base)
    torch.cuda.synchronize()
    diff = (out[:, :, :, -1].float() - od.float()).abs().max().item()
    assert diff <= 0.05, diff
    out2, lse2, _ = _run(q, k, v, wl, 333, base=0.0)
    w = _check(q, k, v, out2, lse2, wl, 333, base=0.0)
    assert w <= TOL_PREFILL


@pytest.mark.parametrize("base", [0.0, 10000.0])
def test_prefill_scores_that_outgrow_the_reference_point(base):
    """Keys whose alignment with the queries grows along the cache: the scores of later tiles exceed the running
    reference point of the softmax by far more than the fp16 range of the weights, so the reference point has
    to move several times (and the weights of the tile that shows it are computed twice).  All operands are
    short binary fractions, so without the rotary embedding the fp16 operands are exact and the scores reach
    tens of units without losing accuracy; with it the keys turn and scores of both signs and all sizes mix."""
    wl = _wl(hkv=2, hq=8, cap=640)
    cur_len, q_len = 600, 333
    k, v = synth.empty_cache(wl, DEV, wl.window)
    k.fill_(float("nan"))
    v.fill_(float("nan"))
    g = torch.Generator(device="cpu").manual_seed(77)
    d = wl.head_dim
    u = (torch.randint(0, 2, (wl.n_heads, d), generator=g) * 2 - 1).float()                 # +-1 per KV head
    ramp = torch.floor(torch.arange(cur_len).float() / cur_len * 256) / 64                  # 0 .. 4 in steps of 1/64
    ramp = ramp * (1 + (torch.arange(cur_len) % 7 == 0).float())                            # with spikes
    kk = u[:, None, :] * ramp[None, :, None]
    k[0, 0, :, :cur_len] = kk.to(torch.bfloat16).to(DEV)
    v[0, 0, :, :cur_len] = torch.randn(wl.n_heads, cur_len, d, generator=g).to(torch.bfloat16).to(DEV)
    # query i of head h: u of its KV head on a random subset of 16..128 channels
    grp = wl.q_heads // wl.n_heads
    keep = torch.rand(wl.q_heads, q_len, d, generator=g) < (torch.randint(1, 9, (wl.q_heads, q_len, 1), generator=g) / 8.0)
    q = (u.repeat_interleave(grp, dim=0)[:, None, :] * keep.float())[None, None].to(torch.bfloat16).to(DEV)
    out, lse, _ = _run(q, k, v, wl, cur_len, base=base)
    # the scaled queries are rounded to fp16: a score of s nats is off by up to s * 2^-11, and lse with it
    # (scores here reach 90 nats, and every channel of a query carries the same rounding error)
    w = _check(q, k, v, out, lse, wl, cur_len, base=base, lse_tol=90 * 2.0 ** -11 + 2e-2)
    _say(f"growing scores, rotary base {base:g}: worst excess / max|V| = {w:.2e}")
    assert w <= TOL_PREFILL


def test_prefill_llama3_chunk_sampled():
    """One layer of the LLaMA-3 shape after a trigger: 4098 compacted rows + a chunk of 4094 tokens = 8192
    cached rows; sampled query rows are checked one by one."""
    wl = _wl(hkv=8, hq=32, layers=1, cap=8192, base=500000.0)
    cur_len, q_len = 8192, 4094
    q, k, v = _mk(wl, cur_len, q_len, seed=8)
    out, lse, p = _run(q, k, v, wl, cur_len)
    rows = [0, 1, 63, 64, 2047, 4000, 4093]
    w = _check(q, k, v, out, lse, wl, cur_len, rows=rows)
    _say(f"prefill 8192/4094: worst excess / max|V| = {w:.2e}  flops {p.flops:.3e}")
    assert w <= TOL_PREFILL


def test_prefill_errors_leave_output_untouched():
    wl = _wl(cap=128)
    q, k, v = _mk(wl, 100, 40, seed=1)
    L = binding.layout_for(k)
    _, p = fk.attend_prefill_plan(L, wl.q_heads, wl.n_heads, 128, 100, 40)
    ws = torch.empty(p.workspace_bytes, dtype=torch.uint8, device=DEV)
    out = torch.full_like(q, 5.0)
    f = lambda *a, **kw: fk.attend_prefill(q, k, v, out, None, L, *a, check=False, **kw)
    assert f(wl.q_heads, wl.n_heads, 128, 100, 40) == -3
    L.workspace, L.workspace_bytes = ws.data_ptr(), p.workspace_bytes
    assert f(wl.q_heads, wl.n_heads, 128, 100, 0) == -1
    assert f(wl.q_heads, wl.n_heads, 128, 100, 101) == -1
    assert f(wl.q_heads, wl.n_heads, 128, 129, 40) == -1
    assert f(wl.q_heads, wl.n_heads, 64, 100, 40) == -2
    assert f(7, wl.n_heads, 128, 100, 40) == -1
    torch.cuda.synchronize()
    assert bool((out == 5.0).all())


def test_prefill_llama2_chunk_sampled():
    """Multi-head attention (one query head per KV head: the four waves of a workgroup take four query
    blocks of different causal reach), LLaMA-2 window: 2050 compacted rows + a chunk of 2046 tokens."""
    wl = synth.small(synth.WORKLOADS["llama2_7b_32k"], n_layers=1, total_tokens=4096)
    cur_len, q_len = 4096, 2046
    q, k, v = _mk(wl, cur_len, q_len, seed=12)
    out, lse, p = _run(q, k, v, wl, cur_len)
    sub = synth.small(wl, n_heads=4)                   # check the first four heads
    w = _check(q[:, :, :4], k[:, :, :4], v[:, :, :4], out[:, :, :4], lse[:, :, :4], sub, cur_len,
               rows=[0, 63, 64, 1000, 2045])
    _say(f"prefill 4096/2046 MHA: worst excess / max|V| = {w:.2e}")
    assert w <= TOL_PREFILL
