#!/usr/bin/env python3
"""Benchmark of the FreqKV compression hot path on one MI355X.

A step = one compression trigger over the whole cache of the workload (all layers' K and V: DCT -> keep the
low half -> inverse -> in-place write, as one factored transform kernel, or fold/convert -> contraction with
--dense) through the C ABI, inputs resident in HBM.
Default workload: the LLaMA-3-8B GQA cache of the 128K iterative prefill (32 layers x 8 KV heads
x head_dim 128, bf16, window 8192, 4 sinks, ratio 0.5): 512 head-tensors, span 8188 -> 4094.

Prints ONE JSON line: whole-job KV-in throughput, the roofline of the dominant kernel (timed by
HIP events on the launch stream inside the library) and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_F16_PEAK_TFLOPS = 2500.0      # MI355X dense fp16/bf16 MFMA
HBM_PEAK_GBS = 8000.0
# HBM bytes (read + write) of the contraction of one trigger (two launches with the two-level fold), from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled by what the same counters read for the library's plain copy
# kernel (profiles/contract_llama3_8b_128k_pmc.txt).
TRAFFIC_BYTES_PER_LAUNCH = {"llama3_8b_128k": (2.0 * (5.244e5 + 9.187e5) + 1.0 * (2.62e5 + 5.24e5)) * 1024}
TRAFFIC_BYTES_SINGLE_FOLD = {"llama3_8b_128k": (2.0 * 2.622e6 + 1.0 * 5.24e5) * 1024}
# the same for the factored transform's single kernel (profiles/fast_llama3_8b_128k_pmc.txt)
FAST_TRAFFIC_BYTES_PER_LAUNCH = {"llama3_8b_128k": (2.0 * 5.4e5 + 1.0 * 5.24e5) * 1024}
# the same for k_attend_partial (profiles/attend_llama3_8b_128k_pmc.txt)
ATTEND_TRAFFIC_BYTES_PER_LAUNCH = {"llama3_8b_128k": (2.0 * 5.248e5 + 1.0 * 1608) * 1024}
# the same for k_attend_prefill (profiles/prefill_llama3_8b_128k.txt)
PREFILL_TRAFFIC_BYTES_PER_LAUNCH = {"llama3_8b_128k": (2.0 * 1.705e6 + 1.0 * 1.049e6) * 1024}


def cpu_baseline(wl, k_cache, cores):
    """The fp64 oracle, as it stands, on `cores` host threads over a bounded sample of head-tensors."""
    import numpy as np
    from oracle import freqkv_oracle as orc
    n_sample = 8 * cores          # about 10-20 s of host work at span 8188
    flat = k_cache.reshape(-1, k_cache.shape[3], k_cache.shape[4])
    idx = [int(i) for i in np.linspace(0, flat.shape[0] - 1, n_sample)]
    heads = [flat[i].to("cpu").float().double().numpy() for i in idx]
    t0 = time.perf_counter()
    orc.compress_heads(heads, wl.window, wl.window, wl.n_sink, wl.retain_ratio, threads=cores)
    dt = time.perf_counter() - t0
    n = wl.window - wl.n_sink
    bytes_in = n_sample * n * wl.head_dim * 2
    return {"value": bytes_in / dt / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"{n_sample} of the workload's head-tensors (K, full span {n} x {wl.head_dim}), "
                      f"{dt:.1f} s on {cores} threads, one head-tensor per thread"}


def attend_cpu_baseline(wl, q, k, v, cores):
    """The fp64 attention oracle on a bounded sample of (layer, batch) slices, one per thread."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from oracle import attend_oracle as att
    n_sample = min(2 * cores, wl.n_layers * wl.batch)
    flat = [(l, b) for l in range(wl.n_layers) for b in range(wl.batch)]
    idx = [flat[int(i)] for i in np.linspace(0, len(flat) - 1, n_sample)]
    data = [(q[l, b].cpu().float().double().numpy(), k[l, b].cpu().float().double().numpy(),
             v[l, b].cpu().float().double().numpy()) for l, b in idx]
    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as ex:
        list(ex.map(lambda a: att.attend_decode(a[0], a[1], a[2], wl.window, None, wl.rope_base), data))
    dt = time.perf_counter() - t0
    bytes_in = n_sample * 2 * wl.n_heads * wl.window * wl.head_dim * 2
    return {"value": bytes_in / dt / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"{n_sample} of the workload's {len(flat)} (layer, batch) slices, all heads, {wl.window} cached rows, "
                      f"{dt:.1f} s on {cores} threads"}


def bench_attend(args, wl, dev):
    """A step = one decode-attention call over every layer's full cache (cur_len = window)."""
    import torch
    import paper_2505_00570_amd as fk
    from paper_2505_00570_amd import binding, synth

    k, v = synth.empty_cache(wl, dev)
    synth.KVSource(wl, seed=0, device=dev).fill(k, v, 0, wl.window)
    q = synth.queries(wl, 0, dev)
    out = torch.empty_like(q)
    lse = torch.empty(q.shape[:3], dtype=torch.float32, device=dev)
    L = binding.layout_for(k)
    _, p = fk.attend_plan(L, wl.q_heads, wl.n_heads, wl.head_dim, wl.window)
    ws = torch.empty(max(p.workspace_bytes, 1 << 30), dtype=torch.uint8, device=dev)
    L.workspace, L.workspace_bytes = ws.data_ptr(), p.workspace_bytes
    stream = torch.cuda.current_stream()

    def step():
        fk.attend_decode(q, k, v, out, lse, L, wl.q_heads, wl.n_heads, wl.head_dim, wl.window, -1, wl.rope_base, stream)

    cpu = None
    if not args.no_cpu_baseline and wl.dtype == torch.bfloat16:
        cpu = attend_cpu_baseline(wl, q, k, v, min(16, os.cpu_count() or 1))
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    fk.profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = fk.profile_read()
    fk.profile_enable(False)
    calib_n = (1 << 29)
    copy_gbs = fk.calibrate_copy(ws[calib_n:].data_ptr(), ws.data_ptr(), calib_n, 10, stream)

    ms_kernel = prof.ms_attend / max(int(prof.launches_attend), 1)
    launches_per_step = max(int(prof.launches_attend), 1) / args.steps
    bytes_launch = p.bytes_algorithmic / launches_per_step
    gbs = bytes_launch / (ms_kernel * 1e-3) / 1e9
    elem = 2 if wl.dtype == torch.bfloat16 else 4
    kv_bytes = 2.0 * wl.n_layers * wl.batch * wl.n_heads * wl.window * wl.head_dim * elem
    out_json = {
        "metric": "decode attention throughput over the compacted cache (GB/s KV read)",
        "value": kv_bytes / (dt / args.steps) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32",
        "dtype_note": "bf16 cache, queries and output; fp32 scores, softmax and accumulation" if elem == 2 else "fp32 throughout",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: decode attention, {wl.n_layers} layers x {wl.batch} x {wl.q_heads} query heads / "
                               f"{wl.n_heads} KV heads x head_dim {wl.head_dim}, {wl.window} cached rows, rotary base "
                               f"{wl.rope_base:g}; one token per sequence per step",
                   "operator": "attend_decode", "n_split": int(p.n_split), "chunk_rows": int(p.chunk_rows),
                   "heads_together": int(p.heads_together)},
        "gflops": p.flops / (dt / args.steps) / 1e9,
        "ms_partial_kernel": ms_kernel,
        "measured_copy_gbs": copy_gbs,
        "roofline": {"bound": "hbm", "kernel": "k_attend_partial", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": gbs / HBM_PEAK_GBS, "traffic": ATTEND_TRAFFIC_BYTES_PER_LAUNCH.get(args.workload),
                     "ms_per_launch": ms_kernel, "bytes_per_launch": bytes_launch, "measured_copy_gbs": copy_gbs,
                     "frac_of_measured_copy": gbs / copy_gbs},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out_json))


def bench_prefill(args, wl, dev):
    """A step = chunk-wise attention of every layer: the chunk that refills the cache after a trigger
    (window - n_sink - Lc tokens) attends to the full cache (cur_len = window)."""
    import torch
    import paper_2505_00570_amd as fk
    from paper_2505_00570_amd import binding, synth

    k, v = synth.empty_cache(wl, dev)
    synth.KVSource(wl, seed=0, device=dev).fill(k, v, 0, wl.window)
    L = binding.layout_for(k)
    _, cp = fk.plan(L, wl.n_heads, wl.head_dim, wl.window, wl.window, wl.n_sink, wl.retain_ratio)
    q_len = wl.window - cp.new_len
    g = torch.Generator(device="cpu").manual_seed(1)
    q = torch.empty(wl.n_layers, wl.batch, wl.q_heads, q_len, wl.head_dim, dtype=torch.bfloat16, device=dev)
    for l in range(wl.n_layers):
        q[l] = (torch.randn(wl.batch, wl.q_heads, q_len, wl.head_dim, generator=g) * 0.5).to(torch.bfloat16).to(dev)
    out = torch.empty_like(q)
    _, p = fk.attend_prefill_plan(L, wl.q_heads, wl.n_heads, wl.head_dim, wl.window, q_len)
    ws = torch.empty(p.workspace_bytes, dtype=torch.uint8, device=dev)
    L.workspace, L.workspace_bytes = ws.data_ptr(), p.workspace_bytes
    stream = torch.cuda.current_stream()

    def step():
        fk.attend_prefill(q, k, v, out, None, L, wl.q_heads, wl.n_heads, wl.head_dim, wl.window, q_len, wl.rope_base, stream)

    cpu = None
    if not args.no_cpu_baseline:
        from concurrent.futures import ThreadPoolExecutor
        from oracle import attend_oracle as att
        cores = min(16, os.cpu_count() or 1)
        rows = [int(i) for i in __import__("numpy").linspace(0, q_len - 1, 4 * cores)]
        kk = k[0, 0, 0].cpu().float().double().numpy()
        vv = v[0, 0, 0].cpu().float().double().numpy()
        qq = q[0, 0, 0].cpu().float().double().numpy()

        def one(i):
            pos = wl.window - q_len + i
            att.attend_decode_head(qq[i], kk, vv, pos + 1, pos, wl.rope_base)
            return 4.0 * wl.head_dim * (pos + 1)

        t0 = time.perf_counter()
        with ThreadPoolExecutor(cores) as ex:
            fl = sum(ex.map(one, rows))
        dtc = time.perf_counter() - t0
        cpu = {"value": fl / dtc / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
               "sample": f"{len(rows)} query rows of one head of layer 0, {dtc:.1f} s on {cores} threads"}
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    fk.profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = fk.profile_read()
    fk.profile_enable(False)
    mfma_tflops = fk.calibrate_mfma(20000, stream)
    launches = max(int(prof.launches_attend), 1)
    ms_kernel = prof.ms_attend / launches
    flops_launch = p.flops * args.steps / launches
    achieved = flops_launch / (ms_kernel * 1e-3) / 1e12
    print(json.dumps({
        "metric": "chunk-wise attention throughput (TFLOP/s, causal flops only)", "value": p.flops / (dt / args.steps) / 1e12,
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "dtype_note": "bf16 cache, queries and output; fp16 MFMA operands, fp32 accumulation and softmax", "data": "synthetic",
        "config": {"workload": f"{wl.name}: chunk-wise attention, {wl.n_layers} layers x {wl.batch} x {wl.q_heads} query heads / "
                               f"{wl.n_heads} KV heads x head_dim {wl.head_dim}, {q_len} chunk tokens over {wl.window} cached rows, "
                               f"rotary base {wl.rope_base:g}", "operator": "attend_prefill"},
        "ms_prepare_kernels": prof.ms_prepare / max(int(prof.launches_prepare), 1), "ms_attend_kernel": ms_kernel,
        "roofline": {"bound": "mfma", "kernel": "k_attend_prefill", "achieved": achieved, "peak": MFMA_F16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / MFMA_F16_PEAK_TFLOPS,
                     "traffic": PREFILL_TRAFFIC_BYTES_PER_LAUNCH.get(args.workload), "ms_per_launch": ms_kernel,
                     "flops_per_launch": flops_launch, "measured_mfma_loop_tflops": mfma_tflops,
                     "frac_of_measured_mfma_loop": achieved / mfma_tflops},
        "cpu_baseline": cpu}))


def bench_e2e(args, wl, dev):
    """A step = the whole iterative prefill of Sec. 3.4 on the KV side: the first window of tokens attends
    causally, then, until total_tokens have streamed through, one compression trigger, the next chunk appended
    behind the compacted rows (a device copy of pre-generated synthetic K/V), chunk-wise attention."""
    import torch
    import paper_2505_00570_amd as fk
    from paper_2505_00570_amd import binding, synth

    k, v = synth.empty_cache(wl, dev)
    src = synth.KVSource(wl, seed=0, device=dev)
    src.fill(k, v, 0, wl.window)
    L = binding.layout_for(k)
    _, cp = fk.plan(L, wl.n_heads, wl.head_dim, wl.window, wl.window, wl.n_sink, wl.retain_ratio)
    chunk = wl.window - cp.new_len
    ck, cv = k[:, :, :, cp.new_len:].clone(), v[:, :, :, cp.new_len:].clone()       # the chunk that is re-appended
    q = (torch.randn(wl.n_layers, wl.batch, wl.q_heads, wl.window, wl.head_dim, device=dev) * 0.5).to(torch.bfloat16)
    out = torch.empty_like(q)
    _, pp = fk.attend_prefill_plan(L, wl.q_heads, wl.n_heads, wl.head_dim, wl.window, wl.window)
    ws = torch.empty(max(pp.workspace_bytes, cp.workspace_bytes), dtype=torch.uint8, device=dev)
    L.workspace, L.workspace_bytes = ws.data_ptr(), ws.numel()
    stream = torch.cuda.current_stream()
    H, d, W = wl.n_heads, wl.head_dim, wl.window

    def step():
        triggers = chunks = 0
        flops = 0.0
        fk.attend_prefill(q, k, v, out, None, L, wl.q_heads, H, d, W, W, wl.rope_base, stream)
        flops += fk.attend_prefill_plan(L, wl.q_heads, H, d, W, W)[1].flops
        done = W
        while done < wl.total_tokens:
            fk.compress(k, v, L, H, d, W, W, wl.n_sink, wl.retain_ratio, stream)
            triggers += 1
            n = min(chunk, wl.total_tokens - done)
            k[:, :, :, cp.new_len:cp.new_len + n].copy_(ck[:, :, :, :n])
            v[:, :, :, cp.new_len:cp.new_len + n].copy_(cv[:, :, :, :n])
            qn = q[:, :, :, :n] if n == W else q.view(-1)[: wl.n_layers * wl.batch * wl.q_heads * n * d].view(
                wl.n_layers, wl.batch, wl.q_heads, n, d)
            on = out.view(-1)[: qn.numel()].view(qn.shape)
            fk.attend_prefill(qn, k, v, on, None, L, wl.q_heads, H, d, cp.new_len + n, n, wl.rope_base, stream)
            flops += fk.attend_prefill_plan(L, wl.q_heads, H, d, cp.new_len + n, n)[1].flops
            chunks += 1
            done += n
        return triggers, chunks, flops

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    fk.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        triggers, chunks, flops = step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    prof = fk.profile_read()
    fk.profile_enable(False)
    ms_compress = (prof.ms_contract + prof.ms_tail) / args.steps
    ms_attend = prof.ms_attend / args.steps
    ms_prepare = prof.ms_prepare / args.steps
    print(json.dumps({
        "metric": "iterative prefill, KV-side path (tokens/s)", "value": wl.total_tokens * wl.batch / dt, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.total_tokens} tokens through a window of {W} ({wl.n_layers} layers, "
                               f"{wl.q_heads}/{H} heads, head_dim {d}): {triggers} compression triggers, "
                               f"{chunks + 1} chunk attentions", "operator": "e2e"},
        "ms_attention_kernels": ms_attend, "ms_contraction_and_tail_kernels": ms_compress,
        "ms_prepare_kernels_both_paths": ms_prepare,
        "compression_share_of_gpu_time": (ms_compress + 0.0) / max(ms_attend + ms_compress + ms_prepare, 1e-9),
        "attention_tflops": flops / (ms_attend * 1e-3) / 1e12,
        "roofline": None, "cpu_baseline": None}))


def bench_spectrum(args, wl, dev):
    """A step = one power-spectrum call over every layer's K and V, all `window` cached rows."""
    import torch
    import paper_2505_00570_amd as fk
    from paper_2505_00570_amd import binding, synth

    k, v = synth.empty_cache(wl, dev)
    synth.KVSource(wl, seed=0, device=dev).fill(k, v, 0, wl.window)
    n = wl.window
    L = binding.layout_for(k)
    _, p = fk.plan(L, wl.n_heads, wl.head_dim, n, n, 0, 0.5)
    ws = torch.empty(p.workspace_bytes + (1 << 20), dtype=torch.uint8, device=dev)
    L.workspace, L.workspace_bytes = ws.data_ptr(), ws.numel()
    out = torch.empty(2, wl.n_layers, wl.n_heads, n, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    def step():
        fk.power_spectrum(k, v, out, L, wl.n_heads, wl.head_dim, 0, n, stream)

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import freqkv_oracle as orc
        x = k[0, :, 0].cpu().float().double().numpy()
        t0 = time.perf_counter()
        orc.power_spectrum(x)
        dtc = time.perf_counter() - t0
        cpu = {"value": x.size * 2 / dtc / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"one (layer, head) of K, {x.shape[0]} sample(s) x {n} rows x {wl.head_dim}, {dtc:.1f} s on 1 thread"}
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    fk.profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = fk.profile_read()
    fk.profile_enable(False)
    mfma_tflops = fk.calibrate_mfma(20000, stream)
    hts = 2 * wl.n_layers * wl.batch * wl.n_heads
    fold = n % 2 == 0
    flops = hts * wl.head_dim * (float(n) * n if fold else 2.0 * n * n)     # executed: the fold halves 2 n^2 d
    launches = max(int(prof.launches_contract), 1)
    ms_contract = prof.ms_contract / launches
    achieved = flops * args.steps / launches / (ms_contract * 1e-3) / 1e12
    bytes_in = hts * n * wl.head_dim * 2
    print(json.dumps({
        "metric": "power-spectrum throughput (GB/s KV in)", "value": bytes_in / (dt / args.steps) / 1e9, "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "dtype_note": "bf16 cache; fp16 MFMA operands, fp32 accumulation and squares", "data": "synthetic",
        "config": {"workload": f"{wl.name}: power spectrum of K and V, {hts} head-tensors x {n} rows x {wl.head_dim}",
                   "operator": "power_spectrum"},
        "ms_prepare_kernel": prof.ms_prepare / max(int(prof.launches_prepare), 1), "ms_contract_kernel": ms_contract,
        "roofline": {"bound": "mfma", "kernel": "k_contract_f16<spectrum>", "achieved": achieved,
                     "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_F16_PEAK_TFLOPS,
                     "traffic": None, "ms_per_launch": ms_contract, "flops_per_launch": flops * args.steps / launches,
                     "measured_mfma_loop_tflops": mfma_tflops, "frac_of_measured_mfma_loop": achieved / mfma_tflops},
        "cpu_baseline": cpu}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama3_8b_128k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", type=int, default=0, help="override the workload's layer count (0: keep)")
    ap.add_argument("--attend", action="store_true",
                    help="time decode attention over the full cache (rotary embedding at read time) instead of compression")
    ap.add_argument("--prefill", action="store_true",
                    help="time chunk-wise attention: a chunk of window - n_sink - Lc queries over the full cache")
    ap.add_argument("--e2e", action="store_true",
                    help="stream the workload's total_tokens through the cache: chunk attention + compression triggers")
    ap.add_argument("--spectrum", action="store_true",
                    help="time the power-spectrum diagnostic over the full window instead of compression")
    ap.add_argument("--single-fold", action="store_true",
                    help="use the one-level even/odd fold where the two-level fold would be chosen (comparison)")
    ap.add_argument("--two-level", action="store_true",
                    help="use the two-level fold wherever it applies, also for spans below its default threshold")
    ap.add_argument("--dense", action="store_true",
                    help="use the matrix form (fp16 MFMA contraction) where the factored transform would be chosen (comparison)")
    ap.add_argument("--stream", action="store_true",
                    help="run the workload's whole trigger schedule (total_tokens through the window), every trigger timed")
    ap.add_argument("--sustain-seconds", type=float, default=2.0,
                    help="length of the sustained loop (triggers with the cache refilled in between); 0 skips it")
    ap.add_argument("--dropping", action="store_true",
                    help="time the Dropping variant (row moves only): the memcpy-roofline reference of the write-back step")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path shards by head with no communication); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2505_00570_amd as fk
    from paper_2505_00570_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    wl = synth.WORKLOADS[args.workload]
    if args.layers > 0:
        wl = synth.small(wl, n_layers=args.layers)
    if args.attend:
        return bench_attend(args, wl, dev)
    if args.spectrum:
        return bench_spectrum(args, wl, dev)
    if args.prefill:
        return bench_prefill(args, wl, dev)
    if args.e2e:
        return bench_e2e(args, wl, dev)

    # synthetic cache, resident in HBM
    k, v = synth.empty_cache(wl, dev)
    synth.KVSource(wl, seed=0, device=dev).fill(k, v, 0, wl.window)
    flags = 0
    if args.dropping:
        flags = fk.FLAG_DROPPING
    elif args.single_fold:
        flags = fk.FLAG_SINGLE_FOLD
    elif args.two_level:
        flags = fk.FLAG_TWO_LEVEL_FOLD
    elif args.dense:
        flags = fk.FLAG_DENSE
    L = binding.layout_for(k, flags=flags)
    _, p = fk.plan(L, wl.n_heads, wl.head_dim, wl.window, wl.window, wl.n_sink, wl.retain_ratio)
    ws = torch.empty(max(p.workspace_bytes, 1 << 30), dtype=torch.uint8, device=dev)     # also the calibration copy's buffer
    L.workspace, L.workspace_bytes = ws.data_ptr(), p.workspace_bytes
    stream = torch.cuda.current_stream()
    H, d, W, S = wl.n_heads, wl.head_dim, wl.window, wl.n_sink

    def step():
        fk.compress(k, v, L, H, d, W, W, S, wl.retain_ratio, stream)

    if args.stream:
        return bench_stream(args, wl, k, v, L, p, step)

    cpu = None
    if not args.no_cpu_baseline and wl.dtype == torch.bfloat16 and not args.dropping:
        cores = min(16, os.cpu_count() or 1)
        cpu = cpu_baseline(wl, k, cores)

    # the rows a caller appends between two triggers (Sec. 3.4: window - n_sink - Lc new tokens), generated once
    chunk_k, chunk_v = k[:, :, :, p.new_len:W].clone(), v[:, :, :, p.new_len:W].clone()

    def refill():
        k[:, :, :, p.new_len:W].copy_(chunk_k)
        v[:, :, :, p.new_len:W].copy_(chunk_v)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- the timed region: K back-to-back triggers on a full cache, inputs resident in HBM
    fk.profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = fk.profile_read()
    fk.profile_enable(False)

    # ---- sustained: at least args.sustain_seconds of triggers, the cache refilled with the pre-generated rows
    # between them (the refill is the caller's work: each trigger is timed by its own pair of events)
    sustained = None
    if args.sustain_seconds > 0 and not args.dropping:
        fk.profile_enable(True)
        evs = []
        t_end = time.perf_counter() + args.sustain_seconds
        while time.perf_counter() < t_end or len(evs) < 8:
            for _ in range(32):
                refill()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(stream)
                step()
                b.record(stream)
                evs.append((a, b))
            torch.cuda.synchronize()
        times = sorted(a.elapsed_time(b) for a, b in evs)
        sprof = fk.profile_read()
        fk.profile_enable(False)
        s_launches = max(int(sprof.launches_contract), 1)
        sustained = {"triggers": len(times), "seconds_of_triggers": sum(times) * 1e-3,
                     "ms_per_step": sum(times) / len(times), "ms_median": times[len(times) // 2],
                     "ms_p10": times[len(times) // 10], "ms_p90": times[len(times) * 9 // 10],
                     "ms_main_kernel_per_trigger": sprof.ms_contract / len(times),
                     "ms_prepare_kernel_per_trigger": sprof.ms_prepare / len(times),
                     "launches_per_trigger": s_launches / len(times)}

    # what this device sustains: plain copy (read+write) and a register-only fp16 MFMA loop on random operands
    calib_n = 1 << 29
    copy_gbs = fk.calibrate_copy(ws[calib_n:].data_ptr(), ws.data_ptr(), calib_n, 10, stream)
    mfma_tflops = fk.calibrate_mfma(20000, stream)

    ms_per_step = dt / args.steps * 1e3
    n = p.span_len
    elem = 2 if wl.dtype == torch.bfloat16 else 4
    bytes_in = p.head_tensors * n * wl.head_dim * elem
    value = bytes_in / (dt / args.steps) / 1e9

    launches = max(int(prof.launches_contract), 1)
    per_trigger = launches / args.steps
    ms_contract = prof.ms_contract / launches
    ms_prepare = prof.ms_prepare / max(int(prof.launches_prepare), 1)
    flops_launch = p.flops_executed * args.steps / launches
    achieved = flops_launch / max(ms_contract * 1e-3, 1e-12) / 1e12
    variant = int(p.variant)
    if args.dropping:
        # the whole step is k_move_rows launches (timed as one span per call by the library)
        ms_move = prof.ms_tail / max(int(prof.calls), 1)
        gbs = p.bytes_algorithmic / (ms_move * 1e-3) / 1e9
        roof = {"bound": "hbm", "kernel": "k_move_rows", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": gbs / HBM_PEAK_GBS, "traffic": None, "ms_per_launch": ms_move,
                "bytes_per_launch": p.bytes_algorithmic, "measured_copy_gbs": copy_gbs,
                "frac_of_measured_copy": gbs / copy_gbs if copy_gbs else None}
    elif variant == 6:
        # the factored transform: one kernel per trigger that reads the span and writes the retained rows; its
        # matrix work is a small fraction of the dense count, so HBM is the roofline it is held against
        bytes_launch = p.bytes_algorithmic / per_trigger
        gbs = bytes_launch / (ms_contract * 1e-3) / 1e9
        roof = {"bound": "hbm", "kernel": "k_fast", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": gbs / HBM_PEAK_GBS, "traffic": FAST_TRAFFIC_BYTES_PER_LAUNCH.get(args.workload),
                "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this kernel (profiles/), "
                                  "not measured by this run",
                "launches_per_trigger": per_trigger, "ms_per_launch": ms_contract, "bytes_per_launch": bytes_launch,
                "measured_copy_gbs": copy_gbs, "frac_of_measured_copy": gbs / copy_gbs,
                "executed_tflops": flops_launch / (ms_contract * 1e-3) / 1e12,
                "sustained_frac": (p.bytes_algorithmic / (sustained["ms_main_kernel_per_trigger"] * 1e-3) / 1e9 / HBM_PEAK_GBS)
                if sustained else None}
    else:
        # the matrix forms: ms_contract is the span of the contraction launches of one pass; the fraction over the
        # whole trigger (prepare pass included) is frac_whole_trigger
        ms_trigger_kernels = (prof.ms_contract + prof.ms_prepare + prof.ms_tail) / args.steps
        roof = {"bound": "mfma", "kernel": "k_contract_f16", "achieved": achieved, "peak": MFMA_F16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / MFMA_F16_PEAK_TFLOPS,
                "frac_whole_trigger": p.flops_executed / (ms_trigger_kernels * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS,
                "traffic": (TRAFFIC_BYTES_SINGLE_FOLD if args.single_fold else TRAFFIC_BYTES_PER_LAUNCH).get(args.workload),
                "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run (profiles/), not measured by this run",
                "launches_per_trigger": 2 if variant == 5 else 1,
                "ms_per_launch": ms_contract, "flops_per_launch": flops_launch,
                "measured_mfma_loop_tflops": mfma_tflops, "frac_of_measured_mfma_loop": achieved / mfma_tflops,
                "sustained_frac": (p.flops_executed / (sustained["ms_main_kernel_per_trigger"] * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS)
                if sustained else None}
    if sustained:
        sustained["value"] = bytes_in / (sustained["ms_per_step"] * 1e-3) / 1e9
        sustained["gbs_algorithmic"] = p.bytes_algorithmic / (sustained["ms_per_step"] * 1e-3) / 1e9

    names = {1: "one-level folded matrix form", 2: "plain matrix form", 3: "fp32 matrix form", 4: "dropping",
             5: "two-level folded matrix form", 6: "factored transform"}
    out = {
        "metric": "KV compression throughput (GB/s KV in)",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if elem == 2 else "f32",
        "dtype_note": "bf16 cache; fp16 MFMA operands, fp32 accumulation" if elem == 2 else "fp32 cache, fp32 FMA",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.n_layers} layers x {wl.batch} x {wl.n_heads} KV heads x "
                               f"head_dim {wl.head_dim}, window {wl.window}, {wl.n_sink} sinks, ratio "
                               f"{wl.retain_ratio}; span {n} -> {p.retained_len}; {p.head_tensors} head-tensors "
                               f"per trigger; one trigger per step",
                   "variant": variant, "form": names.get(variant, "?"),
                   "operator": "dropping" if args.dropping else "freqkv"},
        "tflops_executed": p.flops_executed / (dt / args.steps) / 1e12,
        "tflops_dense_equivalent": p.flops_dense / (dt / args.steps) / 1e12,
        "gbs_algorithmic": p.bytes_algorithmic / (dt / args.steps) / 1e9,
        "frac_hbm_roofline": p.bytes_algorithmic / (dt / args.steps) / 1e9 / HBM_PEAK_GBS,
        "ms_prepare_kernel": ms_prepare, "ms_contract_kernel": ms_contract,
        "measured_copy_gbs": copy_gbs,
        "roofline": roof,
        "sustained": sustained,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


def bench_stream(args, wl, k, v, L, p, step):
    """The whole schedule of the workload (Sec. 3.4): total_tokens streamed through the cache, one trigger each
    time it is full and more tokens arrive; between two triggers the window - n_sink - Lc new rows are written
    from pre-generated rows (they stand for that many decode steps or one prefill chunk).  Every trigger is
    timed by its own pair of events; the refill is not part of the path."""
    import torch
    W, S = wl.window, wl.n_sink
    stream = torch.cuda.current_stream()
    chunk_k, chunk_v = k[:, :, :, p.new_len:W].clone(), v[:, :, :, p.new_len:W].clone()
    free = W - p.new_len
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = []
    fed = W
    while fed < wl.total_tokens:
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        step()
        b.record(stream)
        evs.append((a, b))
        take = min(free, wl.total_tokens - fed)
        k[:, :, :, p.new_len:p.new_len + take].copy_(chunk_k[:, :, :, :take])
        v[:, :, :, p.new_len:p.new_len + take].copy_(chunk_v[:, :, :, :take])
        fed += take
    torch.cuda.synchronize()
    times = sorted(a.elapsed_time(b) for a, b in evs)
    assert len(times) == -(-(wl.total_tokens - W) // free)      # one trigger per refill of the window
    elem = 2 if wl.dtype == torch.bfloat16 else 4
    bytes_in = p.head_tensors * p.span_len * wl.head_dim * elem
    total_ms = sum(times)
    print(json.dumps({
        "metric": "KV compression throughput over the whole schedule (GB/s KV in)",
        "value": bytes_in * len(times) / (total_ms * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": len(times),
        "warmup": args.warmup, "ms_per_step": total_ms / len(times), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.total_tokens} tokens per sequence through a window of {W} "
                               f"({wl.n_layers} layers x {wl.batch} x {wl.n_heads} KV heads x head_dim {wl.head_dim}): "
                               f"{len(times)} triggers of {p.head_tensors} head-tensors, span {p.span_len} -> {p.retained_len}",
                   "variant": int(p.variant), "operator": "freqkv, whole schedule"},
        "triggers": len(times), "ms_median": times[len(times) // 2], "ms_p10": times[len(times) // 10],
        "ms_p90": times[len(times) * 9 // 10], "ms_min": times[0], "ms_max": times[-1],
        "gbs_algorithmic": p.bytes_algorithmic * len(times) / (total_ms * 1e-3) / 1e9,
        "frac_hbm_roofline": p.bytes_algorithmic * len(times) / (total_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "seconds_of_triggers": total_ms * 1e-3, "roofline": None, "cpu_baseline": None}))


if __name__ == "__main__":
    main()
