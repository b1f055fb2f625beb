"""GPU parity of the factored transform (plan variant 6) against the fp64 CPU oracle, element by element.

Spans n = 4pq with a compiled factorization: 140 = 4*5*7 and 1260 = 4*7*45 (small, every head-tensor whole),
4092 = 4*11*93 and 8188 = 4*23*89 (the paper's windows minus 4 sinks).  Same inputs, same tolerance
(tests/_util.py) and same checks as the matrix forms; the oracle runs on the bits the GPU sees.
"""
import math

import numpy as np
import pytest
import torch

import paper_2505_00570_amd as fk
from paper_2505_00570_amd import binding, synth
from oracle import freqkv_oracle as orc

from _util import TOL_BF16, bf16_round, f64, rel_err
from test_gpu_parity import _check_all_heads, _mk, _run, _say

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _wl(layers, batch, heads, d, window, sink=4):
    return synth.small(synth.WORKLOADS["llama2_7b_layer"], n_layers=layers, batch=batch, n_heads=heads, head_dim=d,
                       window=window, n_sink=sink, total_tokens=window)


FAST_SMALL = [
    # (layers, batch, heads, d, window, sink)
    (1, 1, 1, 8, 144, 4),        # n = 140: one task
    (2, 2, 3, 64, 144, 4),       # several layers / sequences / heads, 8 tasks per head-tensor
    (1, 1, 9, 128, 140, 0),      # no sinks; 9 head-tensors per slab: the XCD-aware block map has a remainder
    (1, 1, 2, 128, 1264, 4),     # n = 1260
    (1, 2, 5, 96, 1262, 2),      # head_dim 96, 2 sinks
    (1, 2, 2, 128, 1024, 4),     # n = 1020 = 4*3*85
    (2, 1, 3, 128, 2048, 4),     # n = 2044 = 4*7*73
    (1, 1, 2, 128, 4096, 4),     # n = 4092
    (1, 1, 2, 128, 8192, 4),     # n = 8188
    (1, 1, 1, 256, 8196, 8),     # 8 sinks, head_dim 256
]


@pytest.mark.parametrize("case", FAST_SMALL)
def test_fast_every_element(case):
    layers, batch, heads, d, window, sink = case
    wl = _wl(layers, batch, heads, d, window, sink)
    _say(f"fast variant {case}")
    k, v = _mk(wl, seed=window + d)
    k0, v0 = k.cpu().clone(), v.cpu().clone()
    rc, p, tap = _run(k, v, wl, window)
    assert rc == 0 and p.variant == 6 and p.workspace_bytes == 0
    assert p.retained_len * 2 == p.span_len == window - sink
    _check_all_heads(wl, k0, v0, k.cpu(), v.cpu(), tap.cpu(), p, window, TOL_BF16)


@pytest.mark.parametrize("extra", [1, 17, 700])
def test_fast_tail_and_canaries(extra):
    """cur_len > window: the tail moves bit for bit behind the retained rows, rows beyond cur_len keep
    their canary (both checked inside _check_all_heads)."""
    wl = _wl(1, 2, 2, 128, 1264)
    cur = wl.window + extra
    k, v = _mk(wl, seed=extra, capacity=cur + 5, cur_len=cur)
    k0, v0 = k.cpu().clone(), v.cpu().clone()
    rc, p, tap = _run(k, v, wl, cur)
    assert rc == 0 and p.variant == 6 and p.new_len == 4 + 630 + extra
    _check_all_heads(wl, k0, v0, k.cpu(), v.cpu(), tap.cpu(), p, cur, TOL_BF16)


def test_fast_without_workspace_and_without_tap():
    wl = _wl(1, 1, 3, 128, 1264)
    k, v = _mk(wl, seed=9)
    k0, v0 = k.cpu().clone(), v.cpu().clone()
    L = binding.layout_for(k)                      # workspace NULL: the factored form needs none
    assert fk.compress(k, v, L, wl.n_heads, wl.head_dim, wl.window, wl.window, wl.n_sink, 0.5) == 0
    torch.cuda.synchronize()
    _, p = fk.plan(L, wl.n_heads, wl.head_dim, wl.window, wl.window, wl.n_sink, 0.5)
    _check_all_heads(wl, k0, v0, k.cpu(), v.cpu(), None, p, wl.window, TOL_BF16)


def test_fast_flags_rescale_off_and_dense_agree_with_the_oracle():
    wl = _wl(1, 1, 2, 128, 1264)
    k, v = _mk(wl, seed=21)
    k0, v0 = k.cpu().clone(), v.cpu().clone()
    rc, p, tap = _run(k, v, wl, wl.window, flags=fk.FLAG_NO_RESCALE)
    assert rc == 0 and p.variant == 6
    _check_all_heads(wl, k0, v0, k.cpu(), v.cpu(), tap.cpu(), p, wl.window, TOL_BF16, rescale=False)
    # the matrix form on the same input
    k2, v2 = k0.to(DEV), v0.to(DEV)
    rc, p2, tap2 = _run(k2, v2, wl, wl.window, flags=fk.FLAG_DENSE)
    assert rc == 0 and p2.variant in (1, 5) and p2.workspace_bytes > 0
    _check_all_heads(wl, k0, v0, k2.cpu(), v2.cpu(), tap2.cpu(), p2, wl.window, TOL_BF16)
    # high-frequency retention has no factored form: falls back to the matrix form by itself
    L = binding.layout_for(k, flags=fk.FLAG_RETAIN_HIGH)
    _, p3 = fk.plan(L, wl.n_heads, wl.head_dim, wl.window, wl.window, wl.n_sink, 0.5)
    assert p3.variant in (1, 5)
    # other ratios too
    _, p4 = fk.plan(binding.layout_for(k), wl.n_heads, wl.head_dim, wl.window, wl.window, wl.n_sink, 0.25)
    assert p4.variant in (1, 2, 5)


def test_fast_token_major_strides_and_pointer_table():
    import ctypes as C
    wl = _wl(2, 1, 3, 64, 1264)
    S, W, d, H = wl.n_sink, wl.window, wl.head_dim, wl.n_heads
    # token-major storage [layer][batch][token][head][dim], viewed as [layer][batch][head][token][dim]
    src = synth.KVSource(wl, 31, DEV)
    kk, vv = synth.empty_cache(wl, DEV)
    src.fill(kk, vv, 0, W)
    kt = kk.permute(0, 1, 3, 2, 4).contiguous().permute(0, 1, 3, 2, 4)
    vt = vv.permute(0, 1, 3, 2, 4).contiguous().permute(0, 1, 3, 2, 4)
    assert kt.stride(3) == H * d
    k0, v0 = kt.cpu().clone(), vt.cpu().clone()
    L = binding.layout_for(kt)
    _, p = fk.plan(L, H, d, W, W, S, 0.5)
    assert p.variant == 6
    assert fk.compress(kt, vt, L, H, d, W, W, S, 0.5) == 0
    torch.cuda.synchronize()
    _check_all_heads(wl, k0, v0, kt.cpu(), vt.cpu(), None, p, W, TOL_BF16)
    # per-layer allocations through a host pointer table
    ks = [kk[l:l + 1].clone() for l in range(2)]
    vs = [vv[l:l + 1].clone() for l in range(2)]
    L = binding.layout_for(ks[0])
    L.n_layers, L.pointer_table = 2, 1
    kp = (C.c_void_p * 2)(*[t.data_ptr() for t in ks])
    vp = (C.c_void_p * 2)(*[t.data_ptr() for t in vs])
    assert fk.compress(kp, vp, L, H, d, W, W, S, 0.5) == 0
    torch.cuda.synchronize()
    _check_all_heads(wl, kk.cpu(), vv.cpu(), torch.cat(ks).cpu(), torch.cat(vs).cpu(), None, p, W, TOL_BF16)


@pytest.mark.parametrize("flags", [0, binding.FLAG_DENSE, binding.FLAG_SINGLE_FOLD])
def test_large_and_tiny_values_keep_the_tolerance(flags):
    """Cache values far outside the fp16 range of the matrix-core operands: a K head whose outlier channels
    reach 6e4, a head of magnitude 1e-6, a head of magnitude 3e37 and an all-zero head.  Every head-tensor is
    scaled by an exact power of two on its way in and back on its way out, so none of them overflows to
    inf or drowns in fp16 subnormals."""
    wl = _wl(1, 1, 5, 128, 1264)
    k, v = _mk(wl, seed=77)
    S, W = wl.n_sink, wl.window
    with torch.no_grad():
        k[0, 0, 0, :W] *= 6e4 / float(k[0, 0, 0, :W].abs().float().max())   # its outlier channels reach 6e4
        k[0, 0, 1, :W] *= 1e-6
        v[0, 0, 1, :W] *= 2.0 ** -30
        k[0, 0, 2, :W] *= 3e37 / float(k[0, 0, 2, :W].abs().float().max())
        v[0, 0, 3, :W] = 0
    k0, v0 = k.cpu().clone(), v.cpu().clone()
    rc, p, tap = _run(k, v, wl, W, flags=flags)
    assert rc == 0
    assert torch.isfinite(tap).all()
    _check_all_heads(wl, k0, v0, k.cpu(), v.cpu(), tap.cpu(), p, W, TOL_BF16)
    assert float(v[0, 0, 3, S:S + p.retained_len].abs().max()) == 0.0


def test_fast_stage_one_image_is_the_length_four_butterfly():
    """The diagnostic entry point's image after the load stage: four real p x q arrays per channel --
    sum, alternating sum, and the two differences of the samples j1 = 0..3 of the reordered span --
    times half the power of two that brings the slice's largest magnitude into [256, 512), rows of 96 values
    with their 16-byte chunks rotated against LDS bank conflicts."""
    import ctypes as C
    p_, q_ = 7, 45
    N, n = p_ * q_, 4 * p_ * q_
    wl = _wl(1, 1, 1, 16, n + 4)
    k, v = _mk(wl, seed=3)
    lib = fk.load()
    lib.freqkv_debug_fast_stage.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(binding.Layout), C.c_int, C.c_int,
                                            C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.freqkv_debug_fast_stage.restype = C.c_int
    J2, GH = 8, 96 * 8
    dump = torch.zeros(32 * GH, dtype=torch.float16, device=DEV)
    L = binding.layout_for(k)
    k_before = k.clone()
    assert lib.freqkv_debug_fast_stage(k.data_ptr(), v.data_ptr(), C.byref(L), 1, 16, n + 4, 4, 1, dump.data_ptr(),
                                       dump.numel() * 2, None) == 0
    torch.cuda.synchronize()
    assert torch.equal(k, k_before)                      # the diagnostic writes nothing to the cache
    x = f64(k[0, 0, 0, 4:, :8])
    e = 8 - math.floor(math.log2(np.abs(x).max()))
    phys = dump.double().cpu().numpy().reshape(32 * J2, 12, 8)
    # a row's 12 chunks of 8 values are stored rotated by rot(row) = 2 * bit 2 of the row + bit 3 of the row
    img = np.empty_like(phys)
    for row in range(32 * J2):
        rot = ((row >> 1) & 2) | ((row >> 3) & 1)
        for c in range(12):
            img[row, c] = phys[row, (c + rot) % 12]
    img = img.reshape(4, 8, J2, 96)
    for j2 in range(p_):
        for j3 in range(q_):
            a = []
            for j1 in range(4):
                j = (j1 * N + j2 * 4 * q_ + j3 * 4 * p_) % n
                a.append(x[2 * j if j < n // 2 else 2 * (n - 1 - j) + 1])
            want = np.stack([a[0] + a[1] + a[2] + a[3], a[0] - a[1] + a[2] - a[3], a[0] - a[2], a[3] - a[1]])
            want = want * 0.5 * 2.0 ** e
            got = img[:, :, j2, j3]
            assert np.all(np.abs(got - want) <= 2.0 ** -11 * np.abs(want) + 1e-12), (j2, j3)
    assert np.all(img[:, :, p_:, :] == 0) and np.all(img[:, :, :, q_:] == 0)
