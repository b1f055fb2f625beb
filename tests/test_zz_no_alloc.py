"""freqkv_attend_decode_noalloc (static device scratch, no workspace argument, no allocation) against
freqkv_attend_decode on the same inputs, through the C ABI: the two share their kernels, so the outputs
must be bit-identical.  Two calls in a row, the second on a smaller input (fewer layers, shorter cache),
so a call that leaned on what the previous one left in the shared array would be caught; then the size
limit.  Collected last on purpose."""
import pytest
import torch

import paper_2505_00570_amd as fk
from paper_2505_00570_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _case(layers, batch, hkv, hq, d, cur_len, seed, dtype=torch.bfloat16):
    wl = synth.small(synth.WORKLOADS["llama3_8b_128k"], n_layers=layers, batch=batch, n_heads=hkv, n_q_heads=hq,
                     head_dim=d, window=cur_len, dtype=dtype, total_tokens=cur_len)
    k, v = synth.empty_cache(wl, DEV, cur_len)
    synth.KVSource(wl, seed, DEV).fill(k, v, 0, cur_len)
    q = synth.queries(wl, seed, DEV)
    return wl, q, k, v


def _both(wl, q, k, v, cur_len):
    L = binding.layout_for(k)
    _, p = fk.attend_plan(L, wl.q_heads, wl.n_heads, wl.head_dim, cur_len)
    assert p.workspace_bytes <= fk.noalloc_scratch_bytes()
    ws = torch.empty(max(p.workspace_bytes, 256), dtype=torch.uint8, device=DEV)
    L.workspace, L.workspace_bytes = ws.data_ptr(), p.workspace_bytes
    ref = torch.full_like(q, float("nan"))
    ref_lse = torch.full(q.shape[:3], float("nan"), dtype=torch.float32, device=DEV)
    assert fk.attend_decode(q, k, v, ref, ref_lse, L, wl.q_heads, wl.n_heads, wl.head_dim, cur_len, -1,
                            wl.rope_base) == 0
    L2 = binding.layout_for(k)                      # no workspace at all
    out = torch.full_like(q, float("nan"))
    lse = torch.full_like(ref_lse, float("nan"))
    assert fk.attend_decode_noalloc(q, k, v, out, lse, L2, wl.q_heads, wl.n_heads, wl.head_dim, cur_len, -1,
                                    wl.rope_base) == 0
    torch.cuda.synchronize()
    assert not torch.isnan(ref.float()).any() and not torch.isnan(out.float()).any()
    assert torch.equal(out.view(torch.int16) if out.dtype == torch.bfloat16 else out,
                       ref.view(torch.int16) if ref.dtype == torch.bfloat16 else ref)
    assert torch.equal(lse, ref_lse)
    return p


def test_noalloc_matches_workspace_entry_point_two_calls():
    print("no-alloc attend: 4 layers x 2 seq x (8 q / 2 kv heads) x 4096 rows, then 1 layer x 517 rows", flush=True)
    wl, q, k, v = _case(4, 2, 2, 8, 128, 4096, seed=71)
    p1 = _both(wl, q, k, v, 4096)
    wl2, q2, k2, v2 = _case(1, 1, 2, 4, 128, 517, seed=72)
    p2 = _both(wl2, q2, k2, v2, 517)
    assert p2.workspace_bytes < p1.workspace_bytes
    # and once more on the first, larger input: the array now holds the smaller call's states
    _both(wl, q, k, v, 4096)
    # other head sizes and an fp32 cache go through the same path
    wl3, q3, k3, v3 = _case(2, 1, 4, 4, 64, 300, seed=73, dtype=torch.float32)
    _both(wl3, q3, k3, v3, 300)


def test_noalloc_rejects_what_does_not_fit():
    print("no-alloc attend: size limits", flush=True)
    wl, q, k, v = _case(1, 1, 1, 1, 128, 64, seed=74)
    out = torch.full_like(q, 7.0)
    # more layers than one pass holds: refused before anything is enqueued
    L = binding.layout_for(k)
    L.n_layers = 97
    L.stride_layer = 0
    rc = fk.attend_decode_noalloc(q, k, v, out, None, L, 1, 1, 128, 64, -1, 10000.0, check=False)
    assert rc == binding.E_WORKSPACE and "layers" in fk.last_error()
    # softmax states beyond the static array: 96 layers x 64 sequences x 32 query heads x 128 channels
    L = binding.layout_for(k)
    L.n_layers, L.batch = 96, 64
    L.stride_layer = L.stride_batch = 0
    _, p = fk.attend_plan(L, 32, 1, 128, 64)
    assert p.workspace_bytes > fk.noalloc_scratch_bytes()
    rc = fk.attend_decode_noalloc(q, k, v, out, None, L, 32, 1, 128, 64, -1, 10000.0, check=False)
    assert rc == binding.E_WORKSPACE and "static scratch" in fk.last_error()
    torch.cuda.synchronize()
    assert (out == 7.0).all()
