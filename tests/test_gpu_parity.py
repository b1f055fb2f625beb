"""GPU parity: libfreqkv (HIP, through the C ABI) against the fp64 CPU oracle, element by element.

Inputs are the seeded synthetic tensors of paper_2505_00570_amd.synth; the oracle runs on exactly
the bits the GPU sees (copied to the host before the call).  Tolerances are in tests/_util.py.
"""
import math

import numpy as np
import pytest
import torch

import paper_2505_00570_amd as fk
from paper_2505_00570_amd import binding, synth
from paper_2505_00570_amd.cache import CompressedKVCache
from oracle import freqkv_oracle as orc

from _util import TOL_BF16, TOL_F32, bf16_round, bf16_ulp, f64, rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _say(msg):
    print(msg, flush=True)


def _mk(wl, seed=0, capacity=None, cur_len=None):
    """Cache tensors [L,B,H,cap,d] filled with cur_len synthetic tokens; rows beyond hold a canary."""
    cap = capacity or wl.window
    cur = cur_len or wl.window
    k, v = synth.empty_cache(wl, DEV, cap)
    k.fill_(777.0)
    v.fill_(-777.0)
    synth.KVSource(wl, seed, DEV).fill(k, v, 0, cur)
    return k, v


def _run(k, v, wl, cur_len, tap=True, ws_bytes=None, flags=0, check=True):
    L = binding.layout_for(k, flags=flags)
    _, p = fk.plan(L, wl.n_heads, wl.head_dim, cur_len, wl.window, wl.n_sink, wl.retain_ratio)
    nbytes = p.workspace_bytes if ws_bytes is None else ws_bytes
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=DEV)
    L.workspace, L.workspace_bytes = ws.data_ptr(), nbytes
    tapt = None
    if tap and p.variant != 0:
        tapt = torch.full((2, wl.n_layers, wl.batch, wl.n_heads, p.retained_len, wl.head_dim), float("nan"),
                          dtype=torch.float32, device=DEV)
        L.tap_f32 = tapt.data_ptr()
    rc = fk.compress(k, v, L, wl.n_heads, wl.head_dim, cur_len, wl.window, wl.n_sink, wl.retain_ratio, check=check)
    torch.cuda.synchronize()
    return rc, p, tapt


def _check_all_heads(wl, k0, v0, k1, v1, tap, p, cur_len, tol, rescale=True):
    """Compare every head-tensor with the oracle.  k0/v0: before (host copies), k1/v1: after."""
    S, W, lc = wl.n_sink, wl.window, p.retained_len
    worst_tap, worst_store = 0.0, 0.0
    for kv, (before, after) in enumerate(((k0, k1), (v0, v1))):
        for l in range(wl.n_layers):
            for b in range(wl.batch):
                for h in range(wl.n_heads):
                    x = f64(before[l, b, h, :cur_len])
                    ref = orc.compress_head(x, cur_len, W, S, wl.retain_ratio, rescale=rescale)
                    got = after[l, b, h]
                    # sinks and tail: bit for bit
                    assert torch.equal(got[:S], before[l, b, h, :S])
                    assert torch.equal(got[S + lc:p.new_len], before[l, b, h, W:cur_len])
                    # rows beyond the old cur_len: untouched
                    assert torch.equal(got[cur_len:], before[l, b, h, cur_len:])
                    yref = ref[S:S + lc]
                    rms = max(math.sqrt(float((yref ** 2).mean())), 1e-300)      # an all-zero head must come out all zero
                    ygot = f64(got[S:S + lc])
                    if tap is not None:
                        yt = f64(tap[kv, l, b, h])
                        assert not np.isnan(yt).any()
                        worst_tap = max(worst_tap, rel_err(yt, yref))
                        if wl.dtype == torch.bfloat16:
                            # the stored value is exactly the fp32 result rounded once to bf16
                            assert np.array_equal(ygot, bf16_round(yt))
                        else:
                            assert np.array_equal(ygot, yt)
                    if wl.dtype == torch.bfloat16:
                        # stored bf16: tolerance plus the unavoidable half-ulp of the bf16 grid at |y|
                        excess = np.abs(ygot - yref) - 0.5 * bf16_ulp(yref)
                        worst_store = max(worst_store, float(excess.max()) / rms)
                    else:
                        worst_store = max(worst_store, rel_err(ygot, yref))
    _say(f"  worst fp32-tap err/rms {worst_tap:.3e}  worst stored err/rms (beyond bf16 grid) {worst_store:.3e}")
    assert worst_tap <= tol
    assert worst_store <= tol
    return worst_tap


# ------------------------------------------------------------------------------------------
# config 1: Tiny fp32, full comparison
# ------------------------------------------------------------------------------------------

def test_tiny_fp32_full():
    wl = synth.WORKLOADS["tiny"]
    _say(f"tiny fp32 {wl}")
    k, v = _mk(wl, seed=0)
    k0, v0 = k.cpu().clone(), v.cpu().clone()
    rc, p, tap = _run(k, v, wl, wl.window)
    assert rc == 0 and p.variant == 3 and (p.span_len, p.retained_len) == (508, 254)
    _check_all_heads(wl, k0, v0, k.cpu(), v.cpu(), tap.cpu(), p, wl.window, TOL_F32)


# ------------------------------------------------------------------------------------------
# bf16, small shapes: several tiles, ragged tails, every pipeline tail length, both variants
# ------------------------------------------------------------------------------------------

SMALL = [
    # (layers, batch, heads, d, window, sink, ratio)        what it exercises
    (1, 1, 1, 128, 68, 4, 0.5),      # one pipeline stage (n/2 = 32)
    (1, 1, 2, 128, 132, 4, 0.5),     # two stages
    (1, 1, 1, 128, 196, 4, 0.5),     # three stages
    (1, 1, 1, 128, 260, 4, 0.5),     # four stages
    (1, 1, 1, 128, 330, 4, 0.5),     # six stages, ragged k (n/2 = 163)
    (2, 1, 3, 128, 700, 4, 0.5),     # 11 stages, rows ragged within one tile
    (1, 2, 2, 128, 1300, 4, 0.5),    # rows span two folded tiles (Lc/2 = 324 > 256)
    (1, 1, 2, 128, 701, 4, 0.5),     # odd span -> plain (unfolded) variant
    (1, 1, 1, 128, 1100, 3, 0.5),    # odd span, plain variant, rows span two 512-row tiles? (Lc = 548)
    (1, 1, 3, 64, 516, 4, 0.5),      # head_dim 64: a column tile holds two heads
    (1, 1, 1, 256, 516, 4, 0.5),     # head_dim 256: a head spans two column tiles
    (1, 1, 5, 96, 260, 4, 0.5),      # head_dim 96: column tiles straddle heads, ragged last tile
    (1, 1, 2, 128, 600, 0, 0.25),    # no sinks, ratio 0.25
    (1, 1, 2, 128, 600, 8, 0.75),    # 8 sinks, ratio 0.75
    (1, 1, 2, 128, 600, 2, 0.01),    # ratio 0.01 -> Lc = 5 (odd -> plain)
]

# the two-level fold (default only for long spans), forced on small shapes
TWO_LEVEL = [
    (1, 1, 2, 128, 512, 4, 0.5),     # an odd half: n = 508, Lc = 254, Lc/2 = 127 (a middle row)
    (2, 1, 1, 128, 64, 4, 0.5),      # n = 60, Lc/2 = 15: one stage, almost empty tiles
    (1, 1, 1, 128, 2052, 4, 0.75),   # n = 2048, Lc = 1536: rows of the odd part span two tiles
    (1, 2, 3, 64, 516, 4, 0.5),      # head_dim 64
    (1, 1, 5, 96, 260, 4, 0.5),      # head_dim 96: column tiles straddle heads
    (2, 1, 3, 128, 700, 4, 0.5),     # n = 696, Lc/2 = 174
    (1, 1, 2, 128, 1300, 4, 0.5),    # n = 1296: the even part spans two row tiles
]


@pytest.mark.parametrize("cfg", TWO_LEVEL, ids=[str(c) for c in TWO_LEVEL])
def test_bf16_two_level_fold(cfg):
    layers, batch, heads, d, window, sink, ratio = cfg
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_layers=layers, batch=batch, n_heads=heads, head_dim=d,
                     window=window, n_sink=sink, retain_ratio=ratio)
    _say(f"bf16 two-level {cfg}")
    k, v = _mk(wl, seed=window + d, capacity=window + 7, cur_len=window + 5)
    k0, v0 = k.cpu().clone(), v.cpu().clone()
    rc, p, tap = _run(k, v, wl, window + 5, flags=fk.FLAG_TWO_LEVEL_FOLD)
    assert rc == 0 and p.variant == 5
    _check_all_heads(wl, k0, v0, k.cpu(), v.cpu(), tap.cpu(), p, window + 5, TOL_BF16)



@pytest.mark.parametrize("cfg", SMALL, ids=[str(c) for c in SMALL])
def test_bf16_small_full(cfg):
    nl, b, h, d, W, S, ratio = cfg
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_layers=nl, batch=b, n_heads=h, head_dim=d,
                     window=W, n_sink=S, retain_ratio=ratio, total_tokens=W)
    _say(f"bf16 small {cfg}")
    k, v = _mk(wl, seed=3, capacity=W + 9)
    k0, v0 = k.cpu().clone(), v.cpu().clone()
    rc, p, tap = _run(k, v, wl, W)
    assert rc == 0
    _check_all_heads(wl, k0, v0, k.cpu(), v.cpu(), tap.cpu(), p, W, TOL_BF16)


def test_ratio_one_is_identity():
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_heads=2, window=300, retain_ratio=1.0)
    k, v = _mk(wl, seed=1, capacity=320, cur_len=310)
    k0, v0 = k.clone(), v.clone()
    rc, p, _ = _run(k, v, wl, 310, tap=False)
    assert rc == 0 and p.new_len == 310 and p.variant == 0
    assert torch.equal(k, k0) and torch.equal(v, v0)


def test_noop_below_window_leaves_cache_untouched():
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_heads=2, window=300)
    k, v = _mk(wl, seed=1, capacity=300, cur_len=200)
    k0 = k.clone()
    rc, _, _ = _run(k, v, wl, 200, tap=False)
    assert rc == 1 and torch.equal(k, k0)


# ------------------------------------------------------------------------------------------
# recent tail (cur_len > window), including a tail longer than the freed gap (chunked move)
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("extra", [1, 37, 148, 149, 400])
def test_tail_is_moved_bit_for_bit(extra):
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_layers=2, n_heads=2, window=300, n_sink=4)
    cur = 300 + extra
    _say(f"tail extra={extra}")
    k, v = _mk(wl, seed=5, capacity=cur + 7, cur_len=cur)
    k0, v0 = k.cpu().clone(), v.cpu().clone()
    rc, p, tap = _run(k, v, wl, cur)
    assert rc == 0 and p.new_len == 4 + 148 + extra
    _check_all_heads(wl, k0, v0, k.cpu(), v.cpu(), tap.cpu(), p, cur, TOL_BF16)


# ------------------------------------------------------------------------------------------
# layouts: token-major strides, pointer table, small workspace (several passes)
# ------------------------------------------------------------------------------------------

def test_token_major_strides():
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_layers=2, n_heads=3, window=260)
    W = wl.window
    # storage [L, B, token, H, d] viewed as [L, B, H, token, d]
    ks = torch.empty(2, 1, W, 3, 128, dtype=torch.bfloat16, device=DEV)
    vs = torch.empty_like(ks)
    k, v = ks.permute(0, 1, 3, 2, 4), vs.permute(0, 1, 3, 2, 4)
    synth.KVSource(wl, 2, DEV).fill(k, v, 0, W)
    k0, v0 = k.cpu().clone(), v.cpu().clone()
    rc, p, tap = _run(k, v, wl, W)
    assert rc == 0
    _check_all_heads(wl, k0, v0, k.cpu(), v.cpu(), tap.cpu(), p, W, TOL_BF16)


def test_pointer_table_and_multi_pass_match_single_pass():
    import ctypes as C
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_layers=3, n_heads=2, window=516)
    W = wl.window
    k, v = _mk(wl, seed=9)
    ka, va = k.clone(), v.clone()       # single pass, base pointers
    kb, vb = k.clone(), v.clone()       # minimum workspace -> one slab per pass
    kc, vc = k.clone(), v.clone()       # per-layer pointer table
    rc, p, _ = _run(ka, va, wl, W, tap=False)
    assert rc == 0
    rc, _, _ = _run(kb, vb, wl, W, tap=False, ws_bytes=p.workspace_min_bytes)
    assert rc == 0
    assert torch.equal(ka, kb) and torch.equal(va, vb)
    L = binding.layout_for(kc)
    ws = torch.empty(p.workspace_bytes, dtype=torch.uint8, device=DEV)
    L.workspace, L.workspace_bytes, L.pointer_table = ws.data_ptr(), p.workspace_bytes, 1
    kt = (C.c_void_p * 3)(*[kc[l].data_ptr() for l in range(3)])
    vt = (C.c_void_p * 3)(*[vc[l].data_ptr() for l in range(3)])
    assert fk.compress(kt, vt, L, 2, 128, W, W, 4, 0.5) == 0
    torch.cuda.synchronize()
    assert torch.equal(ka, kc) and torch.equal(va, vc)


def test_errors_leave_memory_untouched():
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_heads=2, window=260)
    k, v = _mk(wl, seed=4)
    k0, v0 = k.clone(), v.clone()
    L = binding.layout_for(k)
    assert fk.compress(k, v, L, 2, 128, 260, 260, 4, 0.5, check=False) == binding.E_WORKSPACE
    rc, _, _ = _run(k, v, wl, 260, tap=False, ws_bytes=64, check=False)
    assert rc == binding.E_WORKSPACE
    L.stride_token = 100
    assert fk.compress(k, v, L, 2, 128, 260, 260, 4, 0.5, check=False) == binding.E_INVALID
    torch.cuda.synchronize()
    assert torch.equal(k, k0) and torch.equal(v, v0)


def test_no_rescale_flag():
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_heads=2, window=260)
    k, v = _mk(wl, seed=6)
    k0, v0 = k.cpu().clone(), v.cpu().clone()
    rc, p, tap = _run(k, v, wl, 260, flags=fk.FLAG_NO_RESCALE)
    assert rc == 0
    _check_all_heads(wl, k0, v0, k.cpu(), v.cpu(), tap.cpu(), p, 260, TOL_BF16, rescale=False)


# ------------------------------------------------------------------------------------------
# iterative schedule (Sec. 3.4): teacher-forced parity at every trigger + free-running drift
# ------------------------------------------------------------------------------------------

def test_iterative_schedule_small():
    wl = synth.small(synth.WORKLOADS["llama2_7b_32k"], n_layers=2, n_heads=2, window=516, total_tokens=516 * 8)
    W, S = wl.window, wl.n_sink
    cache = CompressedKVCache(wl.n_layers, wl.batch, wl.n_heads, wl.head_dim, W, S, wl.retain_ratio, wl.dtype, DEV)
    src = synth.KVSource(wl, 11, DEV)
    lc = cache.plan.retained_len
    free = cache.free_after_trigger
    # free-running fp64 copy of one head-tensor (layer 1, head 1, V)
    fr = None
    fed = 0
    worst = 0.0
    while fed < wl.total_tokens:
        take = min(wl.total_tokens - fed, cache.room() if cache.cur_len < W else free)
        if cache.cur_len >= W:
            before_k = cache.k.cpu().clone()
            before_v = cache.v.cpu().clone()
            assert cache.compress() == 0
            torch.cuda.synchronize()
            after_k = cache.k.cpu()
            for (l, h) in ((0, 0), (1, 1)):
                x = f64(before_k[l, 0, h, :W])
                ref = orc.compress_head(x, W, W, S, wl.retain_ratio)
                got = f64(after_k[l, 0, h, :S + lc])
                rms = math.sqrt(float((ref[S:] ** 2).mean()))
                excess = np.abs(got[S:] - ref[S:]) - 0.5 * bf16_ulp(ref[S:])
                worst = max(worst, float(excess.max()) / rms)
                assert np.array_equal(got[:S], ref[:S])
            if fr is None:
                fr = f64(before_v[1, 0, 1, :W])
            fr = orc.compress_head(fr, W, W, S, wl.retain_ratio)
        kn = torch.empty(wl.n_layers, 1, wl.n_heads, take, wl.head_dim, dtype=wl.dtype, device=DEV)
        vn = torch.empty_like(kn)
        src.fill(kn, vn, 0, take)
        cache.append(kn, vn)
        if fr is not None:
            fr = np.concatenate([fr, f64(vn[1, 0, 1].cpu())])
        fed += take
    assert cache.triggers == orc.trigger_count(wl.total_tokens, W, S, wl.retain_ratio)
    assert worst <= TOL_BF16
    # free-running drift: the bf16 rounding of every earlier trigger is carried along, contracted by
    # sqrt(Lc/n) < 1 per trigger, so it stays within a few half-ulps: allow 5e-2 of the RMS.
    got = f64(cache.v[1, 0, 1, :cache.cur_len].cpu())
    rms = math.sqrt(float((fr ** 2).mean()))
    drift = float(np.max(np.abs(got - fr) - 0.5 * bf16_ulp(fr))) / rms
    _say(f"  triggers {cache.triggers}, teacher-forced worst {worst:.3e}, free-running drift {drift:.3e}")
    assert drift <= 5e-2


# ------------------------------------------------------------------------------------------
# launch plan: more (layer, K|V) slabs than one pointer table holds; caller's stream; helpers
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("window,variant", [(132, 1), (144, 6)])
def test_many_layers_split_into_passes(window, variant):
    """100 layers = 200 slabs > 192 per launch group: the call makes two passes (matrix form and factored form)."""
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_layers=100, n_heads=1, head_dim=64, window=window)
    _say(f"100 layers x 1 head x 64, window {window}")
    k, v = _mk(wl, seed=8, capacity=window + 8)
    k0, v0 = k.cpu().clone(), v.cpu().clone()
    rc, p, tap = _run(k, v, wl, window)
    assert rc == 0 and p.head_tensors == 200 and p.variant == variant
    _check_all_heads(wl, k0, v0, k.cpu(), v.cpu(), tap.cpu(), p, window, TOL_BF16)


@pytest.mark.parametrize("W", [516, 1264])
def test_runs_on_the_callers_stream_and_prepare_is_idempotent(W):
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_heads=2, window=W)
    k, v = _mk(wl, seed=12)
    ka, va = k.clone(), v.clone()
    rc, p, _ = _run(ka, va, wl, W, tap=False)              # default stream
    assert rc == 0
    side = torch.cuda.Stream()
    assert fk.prepare(fk.BF16, 0, W, 4, 0.5, side) == 0     # basis / tables already cached: only a stream wait
    L = binding.layout_for(k)
    ws = torch.empty(max(p.workspace_bytes, 256), dtype=torch.uint8, device=DEV)
    L.workspace, L.workspace_bytes = ws.data_ptr(), p.workspace_bytes
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        assert fk.compress(k, v, L, 2, 128, W, W, 4, 0.5, side) == 0
    side.synchronize()
    assert torch.equal(k, ka) and torch.equal(v, va)        # same bits whichever stream ran it


def test_profile_and_calibration_helpers():
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_heads=4, window=516)
    k, v = _mk(wl, seed=13)
    fk.profile_enable(True)
    for _ in range(3):
        rc, p, _ = _run(k, v, wl, 516, tap=False)
        assert rc == 0
    prof = fk.profile_read()
    fk.profile_enable(False)
    assert prof.calls == 3 and prof.launches_contract == 3 and prof.launches_prepare == 3
    assert prof.launches_tail == 0 and prof.ms_contract > 0 and prof.ms_prepare > 0
    a = torch.empty(1 << 26, dtype=torch.uint8, device=DEV)
    b = torch.randint(0, 255, (1 << 26,), dtype=torch.uint8, device=DEV)
    gbs = fk.calibrate_copy(a, b, 1 << 26, 5)
    assert torch.equal(a, b) and 100.0 < gbs < 16000.0
    tf = fk.calibrate_mfma(2000)
    assert 100.0 < tf < 2600.0
    _say(f"  copy {gbs:.0f} GB/s, mfma loop {tf:.0f} TFLOP/s")


# ------------------------------------------------------------------------------------------
# Dropping variant: pure row moves, bit-exact against the oracle's index rule
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("window,sink,ratio,extra,dtype", [(300, 4, 0.5, 0, torch.bfloat16), (300, 4, 0.75, 0, torch.bfloat16),
                                                           (300, 0, 0.25, 33, torch.bfloat16), (260, 8, 0.9, 400, torch.float32)])
def test_dropping_variant(window, sink, ratio, extra, dtype):
    base = "tiny" if dtype == torch.float32 else "llama2_7b_layer"
    wl = synth.small(synth.WORKLOADS[base], n_layers=2, n_heads=3, head_dim=64, window=window, n_sink=sink,
                     retain_ratio=ratio)
    cur = window + extra
    k, v = _mk(wl, seed=21, capacity=cur + 5, cur_len=cur)
    k0, v0 = k.cpu().clone(), v.cpu().clone()
    L = binding.layout_for(k, flags=fk.FLAG_DROPPING)
    _, p = fk.plan(L, wl.n_heads, wl.head_dim, cur, window, sink, ratio)
    assert p.variant == 4
    assert fk.compress(k, v, L, wl.n_heads, wl.head_dim, cur, window, sink, ratio) == 0   # no workspace needed
    torch.cuda.synchronize()
    for before, after in ((k0, k.cpu()), (v0, v.cpu())):
        for l in range(2):
            for h in range(3):
                ref = orc.drop_head(f64(before[l, 0, h]), cur, window, sink, ratio)
                assert np.array_equal(f64(after[l, 0, h, :p.new_len]), ref)
                assert torch.equal(after[l, 0, h, cur:], before[l, 0, h, cur:])


# ------------------------------------------------------------------------------------------
# batches whose sequences hold different numbers of tokens
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("lens,flags", [([300, 290, 307, 300], 0), ([300, 300, 301, 301], 0), ([10, 299, 0, 42], 0),
                                        ([300, 290, 307, 300], fk.FLAG_DROPPING), ([340, 300, 300, 340], 0),
                                        ([144, 140, 151, 144], 0), ([184, 144, 144, 184], 0)])
def test_ragged_batch(lens, flags):
    window = 144 if max(lens) < 200 else 300             # 144: span 140, the factored form
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_layers=2, batch=4, n_heads=2, window=window)
    cap = window + 60
    _say(f"ragged compress lens={lens} flags={flags}")
    k, v = _mk(wl, seed=77, capacity=cap, cur_len=cap)
    k0, v0 = k.clone(), v.clone()
    L = binding.layout_for(k, flags=flags)
    _, p = fk.plan(L, wl.n_heads, wl.head_dim, wl.window, wl.window, wl.n_sink, wl.retain_ratio)
    ws = torch.empty(max(p.workspace_bytes, 256), dtype=torch.uint8, device=DEV)
    L.workspace, L.workspace_bytes = ws.data_ptr(), p.workspace_bytes
    rc, new_lens = fk.compress_ragged(k, v, L, wl.n_heads, wl.head_dim, lens, wl.window, wl.n_sink, wl.retain_ratio)
    torch.cuda.synchronize()
    assert rc == (0 if any(n >= wl.window for n in lens) else 1)
    for b, n in enumerate(lens):
        assert new_lens[b] == (n if n < wl.window else orc.new_len(n, wl.window, wl.n_sink, wl.retain_ratio))
        if n < wl.window:                                   # not triggered: untouched, bit for bit
            assert torch.equal(k[:, b], k0[:, b]) and torch.equal(v[:, b], v0[:, b])
            continue
        # the same bits as the uniform entry point run on this sequence alone ...
        kb, vb = k0[:, b:b + 1].clone(), v0[:, b:b + 1].clone()
        sub = synth.small(wl, batch=1)
        Lb = binding.layout_for(kb, flags=flags)
        Lb.workspace, Lb.workspace_bytes = ws.data_ptr(), p.workspace_bytes
        fk.compress(kb, vb, Lb, wl.n_heads, wl.head_dim, n, wl.window, wl.n_sink, wl.retain_ratio)
        torch.cuda.synchronize()
        assert torch.equal(k[:, b, :, :new_lens[b]], kb[:, 0, :, :new_lens[b]])
        assert torch.equal(v[:, b, :, :new_lens[b]], vb[:, 0, :, :new_lens[b]])
        assert torch.equal(k[:, b, :, n:], k0[:, b, :, n:])  # rows beyond the old length: untouched
        # ... and, on one head, the oracle directly
        x = f64(k0[1, b, 1, :n].cpu())
        if flags & fk.FLAG_DROPPING:
            ref = orc.drop_head(x, n, wl.window, wl.n_sink, wl.retain_ratio)
            assert np.array_equal(f64(k[1, b, 1, :new_lens[b]].cpu()), ref)
        else:
            ref = orc.compress_head(x, n, wl.window, wl.n_sink, wl.retain_ratio)
            got = f64(k[1, b, 1, :new_lens[b]].cpu())
            S, lc = wl.n_sink, p.retained_len
            rms = math.sqrt(float((ref[S:S + lc] ** 2).mean()))
            excess = np.abs(got[S:S + lc] - ref[S:S + lc]) - 0.5 * bf16_ulp(ref[S:S + lc])
            assert float(excess.max()) / rms <= TOL_BF16
            assert np.array_equal(got[:S], ref[:S]) and np.array_equal(got[S + lc:], ref[S + lc:])


def test_ragged_batch_errors_and_pointer_table():
    import ctypes as C
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_layers=2, batch=3, n_heads=1, window=200)
    k, v = _mk(wl, seed=5, capacity=220, cur_len=220)
    k0 = k.clone()
    L = binding.layout_for(k)
    _, p = fk.plan(L, wl.n_heads, wl.head_dim, wl.window, wl.window, wl.n_sink, wl.retain_ratio)
    ws = torch.empty(p.workspace_bytes, dtype=torch.uint8, device=DEV)
    # a length beyond the capacity anywhere in the batch: nothing is enqueued
    L.workspace, L.workspace_bytes = ws.data_ptr(), p.workspace_bytes
    rc, _ = fk.compress_ragged(k, v, L, wl.n_heads, wl.head_dim, [200, 200, 221], wl.window, wl.n_sink,
                               wl.retain_ratio, check=False)
    assert rc == -1
    L.workspace_bytes = 0
    rc, _ = fk.compress_ragged(k, v, L, wl.n_heads, wl.head_dim, [200, 10, 10], wl.window, wl.n_sink,
                               wl.retain_ratio, check=False)
    assert rc == -3
    rc, nl = fk.compress_ragged(k, v, L, wl.n_heads, wl.head_dim, [199, 10, 10], wl.window, wl.n_sink,
                                wl.retain_ratio, check=False)
    assert rc == 1 and nl == [199, 10, 10]                   # nothing to do needs no workspace
    torch.cuda.synchronize()
    assert torch.equal(k, k0)
    # per-layer pointer table: the runs are addressed through the table
    L.workspace_bytes = p.workspace_bytes
    ref_k, ref_v = k.clone(), v.clone()
    fk.compress_ragged(ref_k, ref_v, binding.layout_for(ref_k, workspace=ws), wl.n_heads, wl.head_dim, [10, 205, 200],
                       wl.window, wl.n_sink, wl.retain_ratio)
    ks = [k[l].clone() for l in range(wl.n_layers)]
    vs = [v[l].clone() for l in range(wl.n_layers)]
    L.pointer_table = 1
    kp = (C.c_void_p * wl.n_layers)(*[t.data_ptr() for t in ks])
    vp = (C.c_void_p * wl.n_layers)(*[t.data_ptr() for t in vs])
    rc, nl = fk.compress_ragged(kp, vp, L, wl.n_heads, wl.head_dim, [10, 205, 200], wl.window, wl.n_sink, wl.retain_ratio)
    torch.cuda.synchronize()
    assert rc == 0
    for l in range(wl.n_layers):
        for b in range(3):
            assert torch.equal(ks[l][b, :, :nl[b]], ref_k[l, b, :, :nl[b]])
            assert torch.equal(vs[l][b, :, :nl[b]], ref_v[l, b, :, :nl[b]])


# ------------------------------------------------------------------------------------------
# high-frequency retention (ablation variant): a different operator through the same kernels
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("window,sink,ratio,extra,dtype", [
    (516, 4, 0.5, 0, torch.bfloat16),      # folded operator (even span, even retained length)
    (1300, 4, 0.5, 9, torch.bfloat16),     # two row tiles, a tail
    (701, 4, 0.5, 0, torch.bfloat16),      # odd span: plain operator, antisymmetric under reversal
    (600, 8, 0.75, 0, torch.bfloat16),
    (600, 2, 0.01, 0, torch.bfloat16),     # five highest coefficients
    (512, 4, 0.5, 0, torch.float32),
])
def test_retain_high_variant(window, sink, ratio, extra, dtype):
    base = synth.WORKLOADS["tiny"] if dtype == torch.float32 else synth.WORKLOADS["llama2_7b_layer"]
    wl = synth.small(base, n_layers=1, batch=1, n_heads=2, window=window, n_sink=sink, retain_ratio=ratio)
    cur = window + extra
    _say(f"retain-high window={window} sink={sink} ratio={ratio} extra={extra} {dtype}")
    k, v = _mk(wl, seed=window, capacity=cur + 3, cur_len=cur)
    if dtype == torch.bfloat16:
        # give the high band something to hold: the synthetic states are low-frequency dominated
        k += (torch.randn(k.shape, device=DEV) * 2.0).to(k.dtype)
        v += (torch.randn(v.shape, device=DEV) * 2.0).to(v.dtype)
    k0, v0 = k.cpu().clone(), v.cpu().clone()
    rc, p, tap = _run(k, v, wl, cur, flags=fk.FLAG_RETAIN_HIGH)
    assert rc == 0
    S, lc = sink, p.retained_len
    worst = 0.0
    for before, after, kv in ((k0, k.cpu(), 0), (v0, v.cpu(), 1)):
        for h in range(wl.n_heads):
            ref = orc.compress_head_high(f64(before[0, 0, h, :cur]), cur, window, sink, ratio)
            got = after[0, 0, h]
            assert torch.equal(got[:S], before[0, 0, h, :S])
            assert torch.equal(got[S + lc:p.new_len], before[0, 0, h, window:cur])
            assert torch.equal(got[cur:], before[0, 0, h, cur:])
            yref = ref[S:S + lc]
            yt = f64(tap[kv, 0, 0, h].cpu())
            worst = max(worst, rel_err(yt, yref))
            if dtype == torch.bfloat16:
                assert np.array_equal(f64(got[S:S + lc]), bf16_round(yt))
            else:
                assert np.array_equal(f64(got[S:S + lc]), yt)
    _say(f"  worst fp32-tap err/rms {worst:.3e}")
    assert worst <= (TOL_BF16 if dtype == torch.bfloat16 else TOL_F32)
    # the flag is part of the basis cache key: the default operator still gives its own result afterwards
    k2, v2 = k0.to(DEV), v0.to(DEV)
    _, _, tap_low = _run(k2, v2, wl, cur)
    ref_low = orc.compress_head(f64(k0[0, 0, 0, :cur]), cur, window, sink, ratio)[S:S + lc]
    assert rel_err(f64(tap_low[0, 0, 0, 0].cpu()), ref_low) <= (TOL_BF16 if dtype == torch.bfloat16 else TOL_F32)


def test_single_fold_flag_matches_two_level_fold():
    """Same operator through the one-level fold (on request) and the two-level fold (default where the span is
    a multiple of 4): both within the tolerance of the oracle, and close to each other."""
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_layers=1, batch=2, n_heads=3, window=1028)
    k, v = _mk(wl, seed=8)
    k1, v1 = k.clone(), v.clone()
    k0 = k.cpu().clone()
    rc, p, tap = _run(k, v, wl, wl.window, flags=fk.FLAG_TWO_LEVEL_FOLD)
    rc1, p1, tap1 = _run(k1, v1, wl, wl.window, flags=fk.FLAG_SINGLE_FOLD)
    assert (p.variant, p1.variant) == (5, 1)
    assert p.flops_executed == pytest.approx(0.75 * p1.flops_executed)
    S, lc = wl.n_sink, p.retained_len
    for h in range(wl.n_heads):
        ref = orc.compress_head(f64(k0[0, 1, h]), wl.window, wl.window, S, wl.retain_ratio)[S:S + lc]
        assert rel_err(f64(tap[0, 0, 1, h].cpu()), ref) <= TOL_BF16
        assert rel_err(f64(tap1[0, 0, 1, h].cpu()), ref) <= TOL_BF16
        assert rel_err(f64(tap[0, 0, 1, h].cpu()), f64(tap1[0, 0, 1, h].cpu())) <= TOL_BF16


def test_retain_high_rejects_dropping():
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_layers=1, n_heads=1, window=100)
    k, v = _mk(wl, seed=1)
    k0 = k.clone()
    L = binding.layout_for(k, flags=fk.FLAG_RETAIN_HIGH | fk.FLAG_DROPPING)
    rc, _ = fk.plan(L, wl.n_heads, wl.head_dim, wl.window, wl.window, wl.n_sink, wl.retain_ratio, check=False)
    assert rc == -1
    rc = fk.compress(k, v, L, wl.n_heads, wl.head_dim, wl.window, wl.window, wl.n_sink, wl.retain_ratio, check=False)
    torch.cuda.synchronize()
    assert rc == -1 and torch.equal(k, k0)


# ------------------------------------------------------------------------------------------
# power-spectrum diagnostic
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("layers,batch,heads,d,row0,n", [
    (1, 1, 1, 128, 0, 256),      # folded transform, one head per column tile
    (2, 3, 2, 128, 4, 508),      # batch averaged into the same lines, sinks skipped
    (1, 2, 3, 64, 0, 330),       # two heads per column tile
    (1, 1, 2, 128, 0, 701),      # odd length: plain transform
    (1, 2, 5, 96, 3, 260),       # column tiles straddle heads
    (1, 1, 2, 128, 0, 2048),     # several row tiles
    (1, 2, 2, 64, 4, -508),      # an fp32 cache (negative n marks it): converted to the same fp16 operands
    (1, 1, 1, 128, 0, -701),     # fp32, odd length
])
def test_power_spectrum(layers, batch, heads, d, row0, n):
    dtype = torch.float32 if n < 0 else torch.bfloat16
    n = abs(n)
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_layers=layers, batch=batch, n_heads=heads, head_dim=d,
                     window=row0 + n, dtype=dtype)
    _say(f"power spectrum layers={layers} batch={batch} heads={heads} d={d} row0={row0} n={n}")
    k, v = _mk(wl, seed=n, capacity=row0 + n + 2, cur_len=row0 + n)
    k0, v0 = k.clone(), v.clone()
    L = binding.layout_for(k)
    _, p = fk.plan(L, heads, d, row0 + n, row0 + n, row0, 0.5)
    ws = torch.empty(p.workspace_bytes + (1 << 16), dtype=torch.uint8, device=DEV)
    L.workspace, L.workspace_bytes = ws.data_ptr(), ws.numel()
    out = torch.full((2, layers, heads, n), float("nan"), dtype=torch.float32, device=DEV)
    fk.power_spectrum(k, v, out, L, heads, d, row0, n)
    torch.cuda.synchronize()
    assert torch.equal(k, k0) and torch.equal(v, v0)            # a diagnostic: the cache is only read
    got = out.cpu().double().numpy()
    worst = 0.0
    for kv, t in enumerate((k0, v0)):
        for l in range(layers):
            for h in range(heads):
                ref = orc.power_spectrum(f64(t[l, :, h, row0:row0 + n].cpu()))
                # fp16 operands: each coefficient carries ~2^-11 relative error plus a floor set by the rounding
                # of the whole span; squaring doubles the relative part
                bound = 5e-3 * ref + 1e-5 * ref.mean()
                err = np.abs(got[kv, l, h] - ref)
                worst = max(worst, float((err / bound).max()))
                # Parseval on the GPU result: the lines sum to the mean energy per channel
                assert math.isclose(got[kv, l, h].sum(), ref.sum(), rel_tol=1e-3)
    _say(f"  worst err/bound {worst:.3f}")
    assert worst <= 1.0
    # twice in a row: the output is overwritten, not accumulated
    fk.power_spectrum(k, v, out, L, heads, d, row0, n)
    torch.cuda.synchronize()
    assert np.allclose(out.cpu().double().numpy(), got, rtol=1e-4, atol=0)


def test_power_spectrum_errors():
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_layers=1, n_heads=1, window=128)
    k, v = _mk(wl, seed=1)
    L = binding.layout_for(k)
    out = torch.full((2, 1, 1, 128), 7.0, dtype=torch.float32, device=DEV)
    f = lambda *a: fk.power_spectrum(k, v, out, L, 1, 128, *a, check=False)
    assert f(0, 128) == -3                      # no workspace
    assert f(0, 129) == -1 and f(-1, 10) == -1 and f(0, 1) == -1
    kf = torch.zeros(1, 1, 1, 128, 128, device=DEV)        # fp32 caches are served too: same workspace rule
    assert fk.power_spectrum(kf, kf, out, binding.layout_for(kf), 1, 128, 0, 128, check=False) == -3
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())


# ------------------------------------------------------------------------------------------
# HIP graph capture: the library only enqueues kernels on the caller's stream (no allocation, no
# memset, no synchronisation once the basis and rotary tables exist), so a trigger followed by decode
# and chunk-wise attention can be captured once and replayed
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("window", [516, 1264])
def test_graph_capture_of_trigger_and_attention(window):
    """Trigger (matrix form at 516, factored form at 1264) + decode attention + chunk attention in one HIP graph."""
    wl = synth.small(synth.WORKLOADS["llama3_8b_128k"], n_layers=2, n_heads=2, n_q_heads=8, window=window)
    k0, v0 = _mk(wl, seed=17)
    k, v = k0.clone(), v0.clone()
    q = synth.queries(wl, 17, DEV)
    L = binding.layout_for(k)
    _, p = fk.plan(L, wl.n_heads, wl.head_dim, wl.window, wl.window, wl.n_sink, wl.retain_ratio)
    _, ap = fk.attend_plan(L, wl.q_heads, wl.n_heads, wl.head_dim, p.new_len)
    q_len = 100                                       # chunk-wise attention of the last 100 compacted rows
    _, pp = fk.attend_prefill_plan(L, wl.q_heads, wl.n_heads, wl.head_dim, p.new_len, q_len)
    ws = torch.empty(max(p.workspace_bytes, ap.workspace_bytes, pp.workspace_bytes), dtype=torch.uint8, device=DEV)
    L.workspace, L.workspace_bytes = ws.data_ptr(), ws.numel()
    out = torch.zeros_like(q)
    g = torch.Generator(device="cpu").manual_seed(18)
    qc = (torch.randn(wl.n_layers, wl.batch, wl.q_heads, q_len, wl.head_dim, generator=g) * 0.5).to(torch.bfloat16).to(DEV)
    outc = torch.zeros_like(qc)

    def work(stream):
        k.copy_(k0)
        v.copy_(v0)
        fk.compress(k, v, L, wl.n_heads, wl.head_dim, wl.window, wl.window, wl.n_sink, wl.retain_ratio, stream)
        fk.attend_decode(q, k, v, out, None, L, wl.q_heads, wl.n_heads, wl.head_dim, p.new_len, -1, wl.rope_base, stream)
        fk.attend_prefill(qc, k, v, outc, None, L, wl.q_heads, wl.n_heads, wl.head_dim, p.new_len, q_len, wl.rope_base, stream)

    # eager reference (also builds the cached basis and rotary tables: the only allocations the library makes)
    work(torch.cuda.current_stream())
    torch.cuda.synchronize()
    k_ref, v_ref, out_ref, outc_ref = k.clone(), v.clone(), out.clone(), outc.clone()
    assert outc_ref.float().abs().max() > 0

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        work(side)                                    # warm-up on the capturing stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            work(torch.cuda.current_stream())
    torch.cuda.synchronize()
    for i in range(4):
        k.zero_(); v.zero_(); out.zero_(); outc.zero_()    # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(k[:, :, :, :p.new_len], k_ref[:, :, :, :p.new_len]), i
        assert torch.equal(v[:, :, :, :p.new_len], v_ref[:, :, :, :p.new_len]), i
        assert torch.equal(out, out_ref), i
        assert torch.equal(outc, outc_ref), i


def test_two_level_fold_in_several_passes():
    """A workspace that holds one (layer, K|V) slab at a time: the two-level fold runs slab by slab, its fp32
    even-part buffer indexed per pass, the optional tap per cache; same bits as the single pass."""
    wl = synth.small(synth.WORKLOADS["llama2_7b_layer"], n_layers=3, batch=2, n_heads=2, window=516)
    k, v = _mk(wl, seed=31, capacity=530, cur_len=523)
    k1, v1 = k.clone(), v.clone()
    L = binding.layout_for(k, flags=fk.FLAG_TWO_LEVEL_FOLD)
    _, p = fk.plan(L, wl.n_heads, wl.head_dim, 523, wl.window, wl.n_sink, wl.retain_ratio)
    assert p.variant == 5 and p.workspace_min_bytes < p.workspace_bytes
    rc, _, tap = _run(k, v, wl, 523, flags=fk.FLAG_TWO_LEVEL_FOLD)
    rc1, _, tap1 = _run(k1, v1, wl, 523, flags=fk.FLAG_TWO_LEVEL_FOLD, ws_bytes=p.workspace_min_bytes)
    assert rc == 0 and rc1 == 0
    assert torch.equal(k, k1) and torch.equal(v, v1) and torch.equal(tap, tap1)
