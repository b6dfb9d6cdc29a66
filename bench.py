#!/usr/bin/env python3
"""Benchmark of the cache-reusing prefill hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input, all inputs resident in HBM:
  query-level match of the batch's query embeddings against the 200k-entry bank  (percache_lookup)
  -> QKV projection + RoPE of the fresh tokens, attention over [cached chunks ; fresh]  (percache_prefill_reuse)
  -> the fresh K/V of every query written into a free slot of the store               (percache_kv_put)
Workload: the 3B-shaped GQA layer, batch 8, 16 cached chunks x 1024 tokens per query gathered from a
1024-slot store, 256 fresh tokens per query (bf16), plus the 200k x 1024 fp16 embedding bank.

Prints ONE JSON line: fresh tokens/s, the roofline of the dominant kernel (reuse attention, bf16 MFMA) from
per-launch HIP-event timings taken inside the timed region, and the CPU oracle timed on a bounded sample.

Timing protocol: W warm-up steps, K steps timed at once (`cold_start`), untimed steps for --settle-ms so that the
clock has settled, then the K timed steps that give `value`.  `warmup` in the line counts every untimed step.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# HBM bytes per launch of the attention kernel on this workload, from rocprofv3 FETCH_SIZE / WRITE_SIZE runs scaled
# by a 1 GiB copy (summary under profiles/).  Valid only for the kernel source the counters were taken with.
ATTN_TRAFFIC = {"source_sha256_16": "e611ef23623c4215", "read_bytes": 2 * 317801.7 * 1024, "write_bytes": 55296.0 * 1024}


def attention_traffic():
    import hashlib
    src = os.path.join(ROOT, "paper_2601_11553_amd", "csrc", "reuse_attention.hip")
    try:
        with open(src, "rb") as f:
            same = hashlib.sha256(f.read()).hexdigest()[:16] == ATTN_TRAFFIC["source_sha256_16"]
    except OSError:
        same = False
    return ATTN_TRAFFIC["read_bytes"] + ATTN_TRAFFIC["write_bytes"] if same else None


def attention_flops(B, Hq, D, T, l_pre):
    """Algorithmic flops of the reuse attention: QK^T and PV over the cached keys and the causal fresh part."""
    return float(sum(4.0 * Hq * D * T * (lp + (T + 1) / 2.0) for lp in l_pre))


def _wall_ms(torch, fn, iters, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    a = time.perf_counter()
    for _ in range(iters):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - a) * 1e3 / iters


def _stats(torch, fn, iters=50, warmup=5):
    """Side-measurement protocol: `iters` (>= 50) calls back to back; per call the GPU time between two events on the
    stream (median and min), and the wall-clock mean over as many calls without events (what a caller's loop sees,
    host launches included)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for e0, e1 in ev:
        e0.record()
        fn()
        e1.record()
    torch.cuda.synchronize()
    a = time.perf_counter()   # (a loop of its own: the event pairs above cost the stream and the host a few us per call)
    for _ in range(iters):
        fn()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - a) * 1e3 / iters
    t = np.array([e0.elapsed_time(e1) for e0, e1 in ev])
    return {"median_ms": round(float(np.median(t)), 4), "min_ms": round(float(t.min()), 4), "wall_mean_ms": round(wall, 4), "iters": iters}


def achievable_peaks(torch, pc, dev):
    """What this GPU sustains with kernels that do nothing else: a register-resident bf16 MFMA loop on constant and on
    random operands, and a streaming read of 1 GiB in which every workgroup walks one contiguous range."""
    res = {}
    for name, rnd in (("mfma_bf16_constant_operands_TFLOPs", False), ("mfma_bf16_random_operands_TFLOPs", True)):
        pc.percache_peak_mfma_bf16(200, rnd)
        torch.cuda.synchronize()
        best = []
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fl = pc.percache_peak_mfma_bf16(20000, rnd)       # about 10-15 ms: long enough for the clock to settle
            e1.record()
            e1.synchronize()
            best.append(fl / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        res[name] = round(float(np.median(best)), 1)
    kv = torch.randn(4 << 20, device=dev).to(torch.bfloat16)      # 8 MiB of N(0,1) values, like the store's contents
    pc.percache_peak_attention_tile_loop(kv, 200)
    torch.cuda.synchronize()
    best = []
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fl = pc.percache_peak_attention_tile_loop(kv, 6000)        # about 10 ms
        e1.record()
        e1.synchronize()
        best.append(fl / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    res["attention_tile_loop_model_TFLOPs"] = round(float(np.median(best)), 1)
    del kv
    buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(3)
    pc.percache_peak_stream_read(buf)
    torch.cuda.synchronize()
    rates = []
    for _ in range(10):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        n = pc.percache_peak_stream_read(buf)
        e1.record()
        e1.synchronize()
        rates.append(n / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    del buf
    res["stream_read_GBps"] = round(float(np.median(rates)), 1)
    return res


def _capture(torch, fn):
    """Captures one call of fn (kernels only) into a HIP graph on a side stream; returns the graph."""
    fn()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        fn()
        graph.capture_end()
    torch.cuda.synchronize()
    return graph


def bench_cfg1(torch, wl, binding, Percache, dev, bf):
    """One 0.6B-shaped layer, batch 1, 4 x 512 cached + 64 fresh tokens: bound by the K/V stream and launch latency.
    Three ways to issue the same call: host chunk lists (a small copy per call), a device-resident chunk table
    (kernels only), and that call captured into a HIP graph and replayed."""
    w = wl.config1()
    pc = Percache(n_layers=1, hidden=w.hidden, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                  n_slots=w.n_slots, slot_capacity=w.chunk_tokens, max_pos=w.max_pos, rope_theta=w.rope_theta, device=dev)
    for s_, (k, v) in w.slots_kv(sorted(set(int(x) for x in w.slot_ids.reshape(-1)))).items():
        pc.percache_kv_put(0, s_, bf(k), bf(v))
    X, W = bf(w.X), bf(w.Wqkv)
    out = torch.empty((1, w.t_fresh, w.n_q_heads * w.head_dim), dtype=torch.bfloat16, device=dev)
    fn = lambda: pc.percache_prefill_reuse(0, X, W, w.slot_ids, w.used_len, attn_out=out)
    table = pc.percache_chunk_table_put(w.slot_ids, w.used_len)
    fn_table = lambda: pc.percache_prefill_reuse_table(0, X, W, table, out)
    _wall_ms(torch, fn, 20, 10)
    ms = _wall_ms(torch, fn, 100, 0)
    pc.percache_profile_enable(True)   # (per-kernel figures from a loop of their own: the event pairs lengthen a call)
    _wall_ms(torch, fn, 100, 0)
    ms_attn, n_attn = pc.percache_profile_read(binding.KERNEL_ATTENTION)
    ms_qkv, n_qkv = pc.percache_profile_read(binding.KERNEL_QKV_ROPE)
    pc.percache_profile_enable(False)
    eager = _stats(torch, fn, 100, 10)
    eager_table = _stats(torch, fn_table, 100, 10)
    graph = _capture(torch, fn_table)
    replay = _stats(torch, graph.replay, 100, 10)
    # GPU time of one call between two events on the stream, caches warm and flushed: for the latter a 512 MiB buffer
    # (twice the last-level cache) is rewritten before each call
    flush = torch.empty(1 << 29, dtype=torch.uint8, device=dev)
    ev = {"warm": [], "cold": []}
    for kind in ("warm", "cold"):
        for _ in range(50):
            if kind == "cold":
                flush.fill_(1)
            torch.cuda._sleep(400_000)   # keeps the GPU busy while the host queues the call: the events then bracket GPU time
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn_table()
            e1.record()
            e1.synchronize()
            ev[kind].append(e0.elapsed_time(e1))
    del flush
    pc.close()
    kv_bytes = float(w.l_pre[0]) * w.n_kv_heads * w.head_dim * 2 * 2
    w_bytes = float(w.Wqkv.size) * 2
    gpu_warm = float(np.median(ev["warm"]))
    return {"ms_per_call": round(ms, 4), "fresh_tokens_per_s": round(w.t_fresh / (ms * 1e-3), 1),
            "host_lists_eager": eager, "device_table_eager": eager_table, "device_table_graph_replay": replay,
            "gpu_ms_per_call_caches_warm": round(gpu_warm, 4), "gpu_ms_per_call_caches_warm_min": round(float(np.min(ev["warm"])), 4),
            "gpu_ms_per_call_caches_flushed": round(float(np.median(ev["cold"])), 4),
            "graph_wall_over_gpu_time": round(replay["wall_mean_ms"] / gpu_warm, 3),
            "attention_ms": round(ms_attn / n_attn, 4), "kv_stream_GBps": round(kv_bytes / (ms_attn / n_attn * 1e-3) / 1e9, 1),
            "qkv_rope_ms": round(ms_qkv / n_qkv, 4), "weight_stream_GBps": round(w_bytes / (ms_qkv / n_qkv * 1e-3) / 1e9, 1)}


def bench_fp8_slots(torch, wl, binding, Percache, dev, bf, w, X, W):
    """The config 4 layer over 8-bit slots (half the store): attention of the 256-token prefill and of one decoding
    token per query over the same 16 chunks."""
    B, T = w.batch, w.t_fresh
    pc = Percache(n_layers=1, hidden=w.hidden, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                  n_slots=w.n_slots, slot_capacity=w.chunk_tokens, max_pos=w.max_pos + 64, rope_theta=w.rope_theta,
                  kv_fp8=True, device=dev)
    for s_, (k, v) in w.slots_kv(sorted(set(int(s) for s in w.slot_ids.reshape(-1)))).items():
        pc.percache_kv_put(0, s_, bf(k), bf(v))
    attn = torch.empty((B, T, w.n_q_heads * w.head_dim), dtype=torch.bfloat16, device=dev)
    attn1 = torch.empty((B, 1, w.n_q_heads * w.head_dim), dtype=torch.bfloat16, device=dev)
    x1 = X[:, :1].contiguous()
    res = {"store_bytes_per_token_and_layer": w.n_kv_heads * w.head_dim * 2 + w.n_kv_heads * 8 // 64,
           "bf16_store_bytes_per_token_and_layer": w.n_kv_heads * w.head_dim * 4}
    for name, fn, iters in (("prefill_attention_ms", lambda: pc.percache_prefill_reuse(0, X, W, w.slot_ids, w.used_len, attn_out=attn), 20),
                            ("decode_attention_ms", lambda: pc.percache_prefill_reuse(0, x1, W, w.slot_ids, w.used_len, attn_out=attn1), 50)):
        _wall_ms(torch, fn, 150, 3)   # (the clock settles under load: the bf16 figures of the step are taken that way too)
        pc.percache_profile_enable(True)
        _wall_ms(torch, fn, max(iters, 50), 0)
        ms, n = pc.percache_profile_read(binding.KERNEL_ATTENTION)
        pc.percache_profile_enable(False)
        res[name] = round(ms / max(n, 1), 4)
    pc.close()
    return res


def bench_cfg2(torch, wl, Percache, dev, bf):
    """28-layer 0.6B-shaped stack: reuse of 8 x 512 cached tokens + 128 fresh rows against the full prefill of all
    4224 tokens (same kernels, no chunks).  The cache is filled by the full pass itself (slicer).  The reuse pass is
    issued with host chunk lists, with a device-resident chunk table, and as a captured HIP graph."""
    w = wl.config2()
    F, L, C, n_c, Tf = 3072, w.n_layers, w.chunk_tokens, w.n_chunks, w.t_fresh
    total = n_c * C + Tf
    pc = Percache(n_layers=L, hidden=w.hidden, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                  n_slots=w.n_slots, slot_capacity=C, max_pos=total, rope_theta=w.rope_theta, device=dev)
    layers = []
    for l in range(L):
        W = wl.stack_weights(2, l, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, F)
        layers.append(dict(gain1=bf(W.gain1), wqkv=bf(W.Wqkv), wo=bf(W.Wo), gain2=bf(W.gain2), w_gate=bf(W.Wgate),
                           w_up=bf(W.Wup), w_down=bf(W.Wdown)))
    h0 = bf(np.random.default_rng(2).standard_normal((1, total, w.hidden)).astype(np.float32))
    slots = [int(x) for x in w.slot_ids[0]]
    bounds = [c * C for c in range(n_c + 1)] + [total]
    h_full = torch.empty_like(h0)
    pc.percache_stack_reuse(layers, F, 1e-6, h0, save_bounds=bounds, save_slots=[slots + [-1]], h_out=h_full)
    hf = h0[:, n_c * C:].contiguous()
    h_reuse = torch.empty_like(hf)
    eager = _stats(torch, lambda: pc.percache_stack_reuse(layers, F, 1e-6, hf, [slots], h_out=h_reuse), 50, 5)
    table = pc.percache_chunk_table_put([slots])
    arr = pc.percache_stack_reuse_table(layers, F, 1e-6, hf, table, h_reuse)
    fn_table = lambda: pc.percache_stack_reuse_table(layers, F, 1e-6, hf, table, h_reuse, weights=arr)
    eager_table = _stats(torch, fn_table, 50, 5)
    graph = _capture(torch, fn_table)
    replay = _stats(torch, graph.replay, 50, 5)
    full = _stats(torch, lambda: pc.percache_stack_reuse(layers, F, 1e-6, h0, h_out=h_full), 50, 2)
    pc.close()
    reuse_ms = min(eager["wall_mean_ms"], eager_table["wall_mean_ms"], replay["wall_mean_ms"])
    return {"reuse_ms": round(reuse_ms, 3), "reuse_host_lists_eager": eager, "reuse_device_table_eager": eager_table,
            "reuse_device_table_graph_replay": replay, "full_recompute": full,
            "full_recompute_ms": full["wall_mean_ms"], "speedup": round(full["wall_mean_ms"] / reuse_ms, 2),
            "fresh_tokens_per_s": round(Tf / (reuse_ms * 1e-3), 1), "layers": L, "cached_tokens": n_c * C, "fresh_tokens": Tf}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--settle-ms", type=float, default=300.0,
                    help="keep the GPU busy with untimed steps for this long before the timed ones (the clock ramps up)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--bank-rows", type=int, default=200_000)
    ap.add_argument("--no-extra", action="store_true", help="skip the config 1 / config 2 side measurements")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (a kernel of known traffic to scale HBM byte counters by)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this library has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2601_11553_amd import workloads as wl
    from paper_2601_11553_amd import binding
    from paper_2601_11553_amd.binding import Percache

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    K_steps = min(args.steps, 256)

    # ------------------------------------------------------------------ inputs (seeded, synthetic)
    w = wl.config4()
    lw = wl.lookup_config3(per_cluster=args.bank_rows // 2000)
    N, d = lw.bank.shape
    B, T = w.batch, w.t_fresh
    n_spare = B
    pc = Percache(n_layers=1, hidden=w.hidden, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                  n_slots=w.n_slots + n_spare, slot_capacity=w.chunk_tokens, max_pos=w.max_pos + 64, rope_theta=w.rope_theta,
                  bank_capacity=N, emb_dim=d, device=dev)
    bf = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(dev, torch.bfloat16)
    used_slots = sorted(set(int(s) for s in w.slot_ids.reshape(-1)))
    for s, (k, v) in w.slots_kv(used_slots).items():
        pc.percache_kv_put(0, s, bf(k), bf(v))
    pc.percache_bank_put(0, torch.from_numpy(lw.bank).to(dev, torch.float16))
    probes_all = torch.from_numpy(lw.probes).to(dev, torch.float16)
    probes = probes_all[:B].contiguous()
    X, W = bf(w.X), bf(w.Wqkv)
    attn = torch.empty((B, T, w.n_q_heads * w.head_dim), dtype=torch.bfloat16, device=dev)
    kf = torch.empty((B, w.n_kv_heads, T, w.head_dim), dtype=torch.bfloat16, device=dev)
    vf = torch.empty_like(kf)
    idx = torch.empty(B, dtype=torch.int32, device=dev)
    sim = torch.empty(B, dtype=torch.float32, device=dev)
    hit = torch.empty(B, dtype=torch.uint8, device=dev)
    spare = [w.n_slots + b for b in range(B)]

    def step():
        pc.percache_lookup(probes, lw.tau, idx, sim, hit)
        pc.percache_prefill_reuse(0, X, W, w.slot_ids, w.used_len, attn_out=attn, k_fresh_out=kf, v_fresh_out=vf)
        pc.percache_kv_put_batch(0, spare, kf, vf, T)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)   # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # The chip raises its clock over the first tens of milliseconds of load and settles after about 0.1 s: K steps
    # timed right after a handful of warm-up steps (12 ms of work at K = 20) run on the ramp and come out about 15 %
    # slower than the same steps a moment later.  Both figures are reported: `cold_start` is exactly W warm-up steps
    # then K timed steps; `value` is K timed steps after further untimed steps have kept the GPU busy for
    # --settle-ms (they are counted in `warmup`).
    t0 = time.perf_counter()
    for _ in range(K_steps):
        step()
    torch.cuda.synchronize()
    cold_ms_step = (time.perf_counter() - t0) * 1e3 / K_steps
    settle_steps = 0
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for _ in range(25):
            step()
        torch.cuda.synchronize()
        settle_steps += 25
    # The timed steps carry the event pair of the roofline's kernel only (a pair costs the stream 2 us: three pairs
    # per step made the step 2 % longer); the other two kernels of the breakdown are timed over K further steps.
    pc.percache_profile_enable(True, kernels=[binding.KERNEL_ATTENTION])
    t0 = time.perf_counter()
    for _ in range(K_steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_attn, n_attn = pc.percache_profile_read(binding.KERNEL_ATTENTION)
    pc.percache_profile_enable(True, kernels=[binding.KERNEL_QKV_ROPE, binding.KERNEL_LOOKUP])
    for _ in range(K_steps):
        step()
    torch.cuda.synchronize()
    ms_qkv, n_qkv = pc.percache_profile_read(binding.KERNEL_QKV_ROPE)
    ms_look, n_look = pc.percache_profile_read(binding.KERNEL_LOOKUP)
    pc.percache_profile_enable(False)
    ms_step = (t1 - t0) * 1e3 / K_steps
    tokens_per_s = B * T / (ms_step * 1e-3)

    # the same step with the bank pass on a second stream of the same priority: the lookup touches only the bank and
    # its own workspace, so it may run beside the prefill (per-kernel figures above come from the serial run)
    side = torch.cuda.Stream()
    ev_fork, ev_join = torch.cuda.Event(), torch.cuda.Event()

    def step_overlapped():
        ev_fork.record()
        with torch.cuda.stream(side):
            side.wait_event(ev_fork)
            pc.percache_lookup(probes, lw.tau, idx, sim, hit)
            ev_join.record()
        pc.percache_prefill_reuse(0, X, W, w.slot_ids, w.used_len, attn_out=attn, k_fresh_out=kf, v_fresh_out=vf)
        pc.percache_kv_put_batch(0, spare, kf, vf, T)
        torch.cuda.current_stream().wait_event(ev_join)

    ms_step_overlapped = _wall_ms(torch, step_overlapped, K_steps, max(args.warmup, 3))
    peaks = achievable_peaks(torch, pc, dev)

    fl_attn = attention_flops(B, w.n_q_heads, w.head_dim, T, w.l_pre)
    attn_ms = ms_attn / max(n_attn, 1)
    attn_tflops = fl_attn / (attn_ms * 1e-3) / 1e12
    fl_qkv = 2.0 * B * T * w.hidden * (w.n_q_heads + 2 * w.n_kv_heads) * w.head_dim
    qkv_ms = ms_qkv / max(n_qkv, 1)
    look_ms = ms_look / max(n_look, 1)
    bank_bytes = N * d * 2 + N * 4
    kv_bytes = float(sum(w.l_pre)) * w.n_kv_heads * w.head_dim * 2 * 2

    # ------------------------------------------------------------------ lookup on its own (lookups/s)
    def time_lookup(p_dev):
        n = p_dev.shape[0]
        oi = torch.empty(n, dtype=torch.int32, device=dev)
        os_ = torch.empty(n, dtype=torch.float32, device=dev)
        oh = torch.empty(n, dtype=torch.uint8, device=dev)
        return _stats(torch, lambda: pc.percache_lookup(p_dev, lw.tau, oi, os_, oh), 50, 3), oh

    look = {}
    for p in (1, 8, 32, 128, 1024):
        st, oh = time_lookup(probes_all[:p].contiguous())
        t = st["median_ms"] * 1e-3
        if p <= 128:  # one streaming pass of the bank (2 N d p flop on N d 2 bytes: below the ridge): HBM bound
            look[f"P{p}"] = dict(st, lookups_per_s=round(p / (st["wall_mean_ms"] * 1e-3), 1), bound="hbm", bank_GBps=round(bank_bytes / t / 1e9, 1),
                                 frac_of_hbm_peak=round(bank_bytes / t / 1e9 / PEAK_HBM_GBS, 4),
                                 frac_of_achievable_stream=round(bank_bytes / t / 1e9 / peaks["stream_read_GBps"], 4))
        else:         # matrix-product kernel: fp16 MFMA bound (2 N d flop per probe)
            tf = 2.0 * N * d * p / t / 1e12
            look[f"P{p}"] = dict(st, lookups_per_s=round(p / (st["wall_mean_ms"] * 1e-3), 1), bound="mfma", TFLOPs=round(tf, 1),
                                 frac_of_fp16_peak=round(tf / PEAK_BF16_TFLOPS, 4),
                                 frac_of_achievable_mfma_random=round(tf / peaks["mfma_bf16_random_operands_TFLOPs"], 4))
            hit_rate = float(oh.float().mean().item())
    # hit rate and the distribution of the gap between the two best similarities of the recipe's 1024 probes
    _, s2 = pc.percache_lookup_topk(probes_all[:1024].contiguous(), 2)
    torch.cuda.synchronize()
    gap = (s2[:, 0] - s2[:, 1]).cpu().numpy()
    edges = [0.0, 1e-4, 1e-3, 1e-2, 1e-1, 2.0]
    hist = np.histogram(gap, bins=edges)[0]
    top1 = s2[:, 0].cpu().numpy()
    # (the recipe's probe noise puts the copies at cosine 0.84, below the recipe's tau: no probe hits at 0.92)
    look["cfg3_probes"] = {"hit_rate_at_tau": round(hit_rate, 4), "tau": lw.tau,
                           "hit_rate_at_other_thresholds": {f"{t:g}": round(float((top1 >= t).mean()), 4) for t in (0.9, 0.85, 0.8, 0.5)},
                           "top2_gap_histogram": {f"[{edges[i]:g},{edges[i + 1]:g})": int(hist[i]) for i in range(len(hist))}}

    # ------------------------------------------------------------------ top-k ranking and the cache refresh scan (same bank)
    p8 = probes_all[:8].contiguous()
    st_topk = _stats(torch, lambda: pc.percache_lookup_topk(p8, 8), 50, 3)
    new64 = probes_all[64:128].contiguous()               # 64 "new chunk" embeddings against every stored row
    kth = torch.full((N,), 0.5, dtype=torch.float32, device=dev)
    st_scan = _stats(torch, lambda: pc.percache_bank_refresh_scan(new64, kth), 50, 3)
    look["topk_P8_k8"] = dict(st_topk, bank_GBps=round(bank_bytes / (st_topk["median_ms"] * 1e-3) / 1e9, 1))
    look["refresh_scan_64_new"] = dict(st_scan, passes_of_the_bank=2, bank_GBps=round(2 * bank_bytes / (st_scan["median_ms"] * 1e-3) / 1e9, 1))

    # ------------------------------------------------------------------ the K/V store itself: 16 whole chunks written / read
    # (their contents are overwritten with other N(0,1) values: nothing after this point compares outputs)
    C = w.chunk_tokens
    some = [int(x) for x in w.slot_ids[0]]
    kc = torch.randn((len(some), w.n_kv_heads, C, w.head_dim), device=dev).to(torch.bfloat16)
    vc = torch.randn_like(kc)
    chunk_bytes = kc.numel() * 2 * 2                                    # K and V
    st_put = _stats(torch, lambda: pc.percache_kv_put_batch(0, some, kc, vc, C), 50, 3)
    ko, vo = torch.empty_like(kc), torch.empty_like(kc)
    st_get = _stats(torch, lambda: pc.percache_kv_get_batch(0, some, C, ko, vo), 50, 3)
    store_io = {"chunks": len(some), "tokens_per_chunk": C, "put_batch": st_put,
                "put_GBps_read_plus_written": round(2 * chunk_bytes / (st_put["median_ms"] * 1e-3) / 1e9, 1),
                "get_batch": st_get, "get_GBps_read_plus_written": round(2 * chunk_bytes / (st_get["median_ms"] * 1e-3) / 1e9, 1)}

    # ------------------------------------------------------------------ one decoding step of the same layer
    # (one new token per query over the 16 reused chunks + the 256-token prompt slot written by the step above)
    x1 = X[:, :1].contiguous()
    ids1 = np.concatenate([w.slot_ids, np.asarray(spare, np.int32)[:, None]], axis=1)
    attn1 = torch.empty((B, 1, w.n_q_heads * w.head_dim), dtype=torch.bfloat16, device=dev)
    dec = lambda: pc.percache_prefill_reuse(0, x1, W, ids1, None, attn_out=attn1)
    st_dec = _stats(torch, dec, 50, 5)
    pc.percache_profile_enable(True)
    dec_ms = _wall_ms(torch, dec, 50, 0)
    dec_attn_ms, dec_n = pc.percache_profile_read(binding.KERNEL_ATTENTION)
    pc.percache_profile_read(binding.KERNEL_QKV_ROPE)
    pc.percache_profile_enable(False)
    dec_bytes = float(B) * (w.l_pre[0] + T) * w.n_kv_heads * w.head_dim * 2 * 2

    out = {
        "metric": "fresh tokens/sec of cache-reuse prefill", "value": round(tokens_per_s, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": K_steps, "warmup": args.warmup + K_steps + settle_steps, "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[4]: 3B-shaped GQA layer (hidden 3072, 24Q/8KV, D128), batch 8, 16x1024 cached "
                               "tokens per query from a 1024-slot store, 256 fresh tokens; step = lookup(8 probes, "
                               f"{N}x{d} fp16 bank) + prefill_reuse + kv_put of fresh K/V",
                   "batch": B, "t_fresh": T, "l_pre": int(w.l_pre[0]), "bank_rows": N},
        "roofline": {"bound": "mfma", "kernel": "reuse_attention_wide_kernel<128>", "achieved": round(attn_tflops, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(attn_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": attention_traffic(), "avg_launch_ms": round(attn_ms, 4), "launches": n_attn,
                     "algorithmic_flops_per_launch": fl_attn, "kv_stream_GBps": round(kv_bytes / (attn_ms * 1e-3) / 1e9, 1),
                     "achievable_peak": peaks,
                     "frac_of_achievable_mfma_random": round(attn_tflops / peaks["mfma_bf16_random_operands_TFLOPs"], 4),
                     "frac_of_achievable_mfma_constant": round(attn_tflops / peaks["mfma_bf16_constant_operands_TFLOPs"], 4),
                     "frac_of_attention_tile_loop_model": round(attn_tflops / peaks["attention_tile_loop_model_TFLOPs"], 4)},
        "cold_start": {"warmup": args.warmup, "steps": K_steps, "ms_per_step": round(cold_ms_step, 4),
                       "value": round(B * T / (cold_ms_step * 1e-3), 1),
                       "note": "the same K steps timed right after W warm-up steps, while the clock still ramps up"},
        "step_variants": {"serial_ms": round(ms_step, 4), "lookup_on_second_stream_ms": round(ms_step_overlapped, 4),
                          "fresh_tokens_per_s_overlapped": round(B * T / (ms_step_overlapped * 1e-3), 1)},
        "breakdown": {
            "qkv_rope": {"avg_launch_ms": round(qkv_ms, 4), "TFLOPs": round(fl_qkv / (qkv_ms * 1e-3) / 1e12, 2),
                         "frac_of_bf16_peak": round(fl_qkv / (qkv_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                         "frac_of_achievable_mfma_random": round(fl_qkv / (qkv_ms * 1e-3) / 1e12 / peaks["mfma_bf16_random_operands_TFLOPs"], 4)},
            "lookup_in_step": {"avg_pass_ms": round(look_ms, 4), "bank_GBps": round(bank_bytes / (look_ms * 1e-3) / 1e9, 1),
                               "frac_of_hbm_peak": round(bank_bytes / (look_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                               "frac_of_achievable_stream": round(bank_bytes / (look_ms * 1e-3) / 1e9 / peaks["stream_read_GBps"], 4)},
            "lookup_alone": look,
            "kv_store_io": store_io,
            "decode_step_layer": {"ms_per_call": round(dec_ms, 4), "per_call": st_dec, "attention_ms": round(dec_attn_ms / max(dec_n, 1), 4),
                                  "kv_stream_GBps": round(dec_bytes / (dec_attn_ms / max(dec_n, 1) * 1e-3) / 1e9, 1),
                                  "keys_per_query": int(w.l_pre[0] + T), "batch": B},
        },
    }

    # ------------------------------------------------------------------ side measurements: config 1 layer, config 2 stack
    if not args.no_extra:
        pc.close()
        del pc
        torch.cuda.empty_cache()
        pc = None
        # (side measurements: one that fails is reported as such and does not take the step's figures with it)
        for name, fn in (("cfg4_layer_8bit_slots", lambda: bench_fp8_slots(torch, wl, binding, Percache, dev, bf, w, X, W)),
                         ("cfg1_layer", lambda: bench_cfg1(torch, wl, binding, Percache, dev, bf)),
                         ("cfg2_stack", lambda: bench_cfg2(torch, wl, Percache, dev, bf))):
            try:
                out["breakdown"][name] = fn()
            except Exception as e:  # noqa: BLE001
                out["breakdown"][name] = {"error": f"{type(e).__name__}: {e}"}
            torch.cuda.empty_cache()

    # ------------------------------------------------------------------ CPU oracle on a bounded sample
    if not args.no_cpu_baseline:
        import oracle
        nthreads = oracle.num_threads()
        # whole queries of the same batch, one after the other, until about 10 s of projection + attention are spent
        t_proj = t_attn = 0.0
        n_q = 0
        for b in range(B):
            sk, sv, ids = w.compact_store(b)
            a = time.perf_counter()
            Qo, Ko, Vo = oracle.qkv_rope(w.X[b], w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, int(w.l_pre[b]), w.rope_theta)
            t_proj += time.perf_counter() - a
            a = time.perf_counter()
            oracle.attention_reuse(Qo, Ko, Vo, sk, sv, ids, w.used_len[b])
            t_attn += time.perf_counter() - a
            n_q += 1
            if t_proj + t_attn > 10.0:
                break
        # lookups: a pilot of 16 probes sizes a sample of about 5 s
        a = time.perf_counter()
        oracle.lookup(lw.bank, lw.probes[:16], lw.tau)
        t_pilot = time.perf_counter() - a
        n_look_cpu = int(min(lw.probes.shape[0], max(16, 5.0 / max(t_pilot / 16, 1e-6))))
        a = time.perf_counter()
        oracle.lookup(lw.bank, lw.probes[:n_look_cpu], lw.tau)
        t_look = time.perf_counter() - a
        per_query = (t_proj + t_attn) / n_q + t_look / n_look_cpu
        out["cpu_baseline"] = {
            "value": round(T / per_query, 2), "unit": "tokens/s", "cores": nthreads, "kind": "oracle",
            "cores_in_affinity_mask": len(os.sched_getaffinity(0)), "openmp_threads": nthreads,
            "sample": f"the first {n_q} of the {B} queries of the same workload in full (projection+RoPE of {T} fresh tokens "
                      f"{t_proj:.2f} s, attention of {T} rows x {w.n_q_heads} heads over {int(w.l_pre[0])} cached + fresh keys "
                      f"{t_attn:.2f} s) and the lookup of {n_look_cpu} probes against the {N}-row bank ({t_look:.2f} s); "
                      f"value = {T} tokens / (prefill seconds per query + lookup seconds per probe)",
        }
    print(json.dumps(out))
    if pc is not None:
        pc.close()


if __name__ == "__main__":
    main()
